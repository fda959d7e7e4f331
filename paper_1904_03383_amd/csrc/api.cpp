// Host side of the tgemm C-ABI (include/tgemm.h): argument validation, choice of a
// tile configuration (forced > tuned > static heuristic), the timing tuner with its
// lower-bound pruning, the tune cache, and kernel dispatch.  No device memory is
// allocated or freed here.
#include "tg_internal.h"

#include "../../include/tgemm.h"

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <initializer_list>
#include <map>
#include <mutex>
#include <string>
#include <tuple>
#include <vector>

namespace {

using tg::GemmParams;
using tg::KernelInfo;

constexpr int kVersion = 100;               // 0.1.0
constexpr int kNumCUs = 256;                // MI355X: 8 XCDs x 32 CUs
constexpr double kPeakFlops = 157.3e12;     // fp32 MFMA: 256 CU x 256 flop/clk x 2.4 GHz
constexpr double kPeakHbm = 8.0e12;         // bytes/s
constexpr double kSimdFlops = 64 * 2.4e9;   // one SIMD: 64 flop/clk
constexpr int kLongK = 1024;                // K range above which second-level accumulators are required
constexpr int kFlushK = 1024;               // K terms between folds of the first-level accumulators (measured at 4096^3:
                                            // 512 -> 4.1e-7 relative Frobenius error, 1024 -> 5.7e-7 and 0.5 % faster,
                                            // 2048 -> 8.1e-7, never -> 1.15e-6)
constexpr int kLongKPieces = 8192;          // longest K range of the bf16-piece kernels: their leading chain rounds once per
                                            // 16 terms, so 8192 terms are 512 roundings (4096 terms measured: 3.9e-7)
constexpr int kWaveMaxK = 2048;             // longest K the single-accumulator wave kernel may take
constexpr int kDefaultGroup = 8;
using tg::kLdsPerCU;

thread_local std::string t_error;
thread_local std::string t_last_config;

struct Config {
    int kernel = -1;
    int splits = 1;
    int group = kDefaultGroup;
    int occ = 0;   // cap on workgroups per CU (0 = whatever fits)
    int persist = 0;   // > 0: persistent launch with this many workgroups per CU
    // Tail split: the last `tail` tile rows of every problem go out as a second launch with split-K
    // `tail_splits`, so that a tile count just above a multiple of what the chip holds does not cost a
    // whole extra round of workgroups (0 = one launch).
    int tail = 0;
    int tail_splits = 1;
};

// What tg_last_config() reports: the spec string is formatted on demand from the last call's choice.
thread_local Config t_last_cfg;
thread_local const char *t_last_tags[2] = {"", ""};   // "+pack..." and "+align..." suffixes (string literals)
thread_local bool t_last_pending = false;

struct Problem {
    int64_t batch, m, n, k;
    const float *A; int64_t lda, strideA;
    const float *B; int64_t ldb, strideB;
    float *C; int64_t ldc, strideC;
    bool aligned;   // every row of A and B (and every problem) starts on a 16-byte boundary, unit element strides
                    // (C's alignment only decides between vector and element stores)
    int64_t csa = 1, csb = 1;   // element strides along k of A / along n of B (strided entry point)
    int64_t nb = 0;             // columns of B the exact-fit kernels may fetch (0: n); n rounded up to 4 for a padded copy
    bool a_al = true, b_al = true;   // base (and batch stride) of A / B on the 16-byte grid (set by validate)
    int64_t b_cols() const { return nb ? nb : n; }
    bool unit() const { return csa == 1 && csb == 1; }
    // Can a kernel that reads A / B in this operand mode take the operand as it lies?  (KernelInfo::amode, bmode:
    // 0 plain with 16-byte rows, 1 transposed with 16-byte rows, 2 any element strides)
    bool a_fits(int mode) const {
        if (mode == 0) return csa == 1 && a_al && lda % 4 == 0;
        if (mode == 1) return lda == 1 && csa % 4 == 0 && a_al && m % 4 == 0;
        return true;
    }
    bool b_fits(int mode) const {
        if (mode == 0) return csb == 1 && b_al && ldb % 4 == 0;
        if (mode == 1) return ldb == 1 && csb % 4 == 0 && b_al;
        return true;
    }
    int a_class() const { return a_fits(0) ? 0 : (a_fits(1) ? 1 : 2); }
    int b_class() const { return b_fits(0) ? 0 : (b_fits(1) ? 1 : 2); }
};

typedef std::tuple<int64_t, int64_t, int64_t, int64_t, int> ShapeKey;

struct TunedEntry {
    Config cfg;
    double usec;
};

std::mutex g_mutex;
std::map<ShapeKey, TunedEntry> g_cache;
std::map<std::pair<ShapeKey, size_t>, Config> g_heuristic_choice;   // memo of the static heuristic
void *g_ws = nullptr;
size_t g_ws_bytes = 0;
bool g_forced = false;
std::atomic<int> g_math{TG_MATH_FP32_MFMA};   // which arithmetic the automatic choice may use (read by the tuner without the lock)
bool g_env_read = false;
Config g_force_cfg;
int g_device_ok[64] = {0};  // 0 unknown, 1 gfx950, -1 other

tg_status fail(tg_status s, const std::string &msg) {
    t_error = msg;
    return s;
}

std::string spec_of(const Config &c) {
    char buf[160];
    int n = snprintf(buf, sizeof buf, "%s:s%d:g%d", tg::kernel(c.kernel).name, c.splits, c.group);
    if (c.occ > 0) n += snprintf(buf + n, sizeof buf - n, ":o%d", c.occ);
    if (c.persist > 0) n += snprintf(buf + n, sizeof buf - n, ":p%d", c.persist);
    if (c.tail > 0) n += snprintf(buf + n, sizeof buf - n, ":t%dx%d", c.tail, c.tail_splits);
    return buf;
}

int find_kernel(const std::string &name) {
    for (int i = 0; i < tg::num_kernels(); ++i)
        if (name == tg::kernel(i).name) return i;
    return -1;
}

// "<kernel>[:s<splits>][:g<group>][:o<cap on workgroups per CU>][:p<persistent workgroups per CU>][:t<tail tile rows>x<tail splits>]"
bool parse_spec(const char *spec, Config &out, std::string &why) {
    std::string s(spec);
    size_t pos = s.find(':');
    std::string name = s.substr(0, pos);
    Config c;
    c.kernel = find_kernel(name);
    if (c.kernel < 0) { why = "unknown kernel '" + name + "'"; return false; }
    while (pos != std::string::npos) {
        size_t next = s.find(':', pos + 1);
        std::string tok = s.substr(pos + 1, next == std::string::npos ? std::string::npos : next - pos - 1);
        if (tok.size() < 2 || (tok[0] != 's' && tok[0] != 'g' && tok[0] != 'o' && tok[0] != 'p' && tok[0] != 't')) { why = "bad token '" + tok + "'"; return false; }
        char *end = nullptr;
        long v = strtol(tok.c_str() + 1, &end, 10);
        if (tok[0] == 't') {   // t<rows>x<splits>
            if (*end != 'x' || v < 1 || v > 4096) { why = "bad value in '" + tok + "'"; return false; }
            char *end2 = nullptr;
            const long v2 = strtol(end + 1, &end2, 10);
            if (end2 == end + 1 || *end2 != '\0' || v2 < 2 || v2 > 4096) { why = "bad value in '" + tok + "'"; return false; }
            c.tail = (int)v;
            c.tail_splits = (int)v2;
            pos = next;
            continue;
        }
        if (*end != '\0' || v < 1 || v > 4096) { why = "bad value in '" + tok + "'"; return false; }
        if (tok[0] == 's') c.splits = (int)v;
        else if (tok[0] == 'g') c.group = (int)v;
        else if (tok[0] == 'o') c.occ = (int)v;
        else c.persist = (int)v;
        pos = next;
    }
    out = c;
    return true;
}

// Tune cache file: plain text, one entry per line.  Callers hold g_mutex.
tg_status save_cache_locked(const char *path) {
    FILE *f = fopen(path, "w");
    if (!f) return fail(TG_ERR_INVALID_ARG, std::string("cannot open ") + path + " for writing");
    fprintf(f, "tgemm-tune-cache 5 gfx950\n");
    for (const auto &kv : g_cache) {
        const ShapeKey &k = kv.first;
        fprintf(f, "%lld %lld %lld %lld %d %s %d %d %d %d %d %d %.3f\n", (long long)std::get<0>(k), (long long)std::get<1>(k),
                (long long)std::get<2>(k), (long long)std::get<3>(k), std::get<4>(k),
                tg::kernel(kv.second.cfg.kernel).name, kv.second.cfg.splits, kv.second.cfg.group, kv.second.cfg.occ,
                kv.second.cfg.persist, kv.second.cfg.tail, kv.second.cfg.tail_splits, kv.second.usec);
    }
    fclose(f);
    return TG_OK;
}

tg_status load_cache_locked(const char *path) {
    FILE *f = fopen(path, "r");
    if (!f) return fail(TG_ERR_INVALID_ARG, std::string("cannot open ") + path);
    char head[64] = {0}, arch[32] = {0};
    int ver = 0;
    if (fscanf(f, "%63s %d %31s", head, &ver, arch) != 3 || strcmp(head, "tgemm-tune-cache") != 0 || (ver < 3 || ver > 5) ||
        strcmp(arch, "gfx950") != 0) {
        fclose(f);
        return fail(TG_ERR_INVALID_ARG, "not a tgemm tune cache for gfx950 (version 3 to 5)");
    }
    // one entry per line; version 4 added the two tail-split fields before the time, version 5 widened the
    // layout class (the math mode moved from 4 x to 16 x)
    char line[512];
    while (fgets(line, sizeof line, f)) {
        long long b, m, n, k;
        int al, splits, group, occ, persist, tail = 0, tail_splits = 1;
        char name[128];
        double us;
        int got;
        if (ver == 3)
            got = sscanf(line, "%lld %lld %lld %lld %d %127s %d %d %d %d %lf", &b, &m, &n, &k, &al, name, &splits, &group, &occ,
                         &persist, &us) == 11;
        else
            got = sscanf(line, "%lld %lld %lld %lld %d %127s %d %d %d %d %d %d %lf", &b, &m, &n, &k, &al, name, &splits, &group,
                         &occ, &persist, &tail, &tail_splits, &us) == 13;
        if (!got) continue;
        Config c;
        c.kernel = find_kernel(name);
        c.splits = splits;
        c.group = group;
        c.occ = occ;
        c.persist = persist;
        c.tail = tail;
        c.tail_splits = tail_splits;
        // entry from another build or a damaged line: ignore
        if (c.kernel < 0 || splits < 1 || group < 1 || occ < 0 || persist < 0 || tail < 0 || tail_splits < 1) continue;
        if (ver < 5) al = al % 4 + 16 * (al / 4);
        g_cache[ShapeKey(b, m, n, k, al)] = TunedEntry{c, us};
    }
    fclose(f);
    return TG_OK;
}

void read_env_once() {
    if (g_env_read) return;
    g_env_read = true;
    // TG_TUNE_CACHE: a tune cache file that is loaded now (if it exists) and rewritten after every tg_tune
    if (const char *path = getenv("TG_TUNE_CACHE")) {
        if (*path) {
            FILE *probe = fopen(path, "r");
            if (probe) {
                fclose(probe);
                if (load_cache_locked(path) != TG_OK) fprintf(stderr, "tgemm: ignoring TG_TUNE_CACHE: %s\n", t_error.c_str());
            }
        }
    }
    const char *e = getenv("TG_FORCE_CONFIG");
    if (e && *e) {
        Config c;
        std::string why;
        if (parse_spec(e, c, why)) { g_forced = true; g_force_cfg = c; }
        else fprintf(stderr, "tgemm: ignoring TG_FORCE_CONFIG: %s\n", why.c_str());
    }
}

bool mul_ovf(int64_t a, int64_t b, int64_t *r) { return __builtin_mul_overflow(a, b, r); }
bool add_ovf(int64_t a, int64_t b, int64_t *r) { return __builtin_add_overflow(a, b, r); }

// extent of a strided matrix: (rows-1)*ld + cols, false on overflow
bool extent(int64_t rows, int64_t cols, int64_t ld, int64_t *out) {
    if (rows == 0 || cols == 0) { *out = 0; return true; }
    int64_t t;
    if (mul_ovf(rows - 1, ld, &t)) return false;
    return !add_ovf(t, cols, out);
}

tg_status validate(Problem &p) {
    if (p.batch < 0 || p.m < 0 || p.n < 0 || p.k < 0)
        return fail(TG_ERR_INVALID_ARG, "negative size");
    if (p.unit()) {
        if (p.lda < std::max<int64_t>(p.k, 1) || p.ldb < std::max<int64_t>(p.n, 1))
            return fail(TG_ERR_INVALID_ARG, "leading dimension too small: need lda >= max(k,1), ldb >= max(n,1), ldc >= max(n,1)");
    } else if (p.lda < 1 || p.ldb < 1 || p.csa < 1 || p.csb < 1) {
        return fail(TG_ERR_INVALID_ARG, "element strides of A and B must be positive");
    }
    if (p.ldc < std::max<int64_t>(p.n, 1))
        return fail(TG_ERR_INVALID_ARG, "leading dimension too small: need lda >= max(k,1), ldb >= max(n,1), ldc >= max(n,1)");
    if (p.strideA < 0 || p.strideB < 0 || p.strideC < 0)
        return fail(TG_ERR_INVALID_ARG, "negative batch stride");
    int64_t ea, eb, ec, t;
    if (!extent(p.m, p.k, p.lda, &ea) || !extent(p.k, p.n, p.ldb, &eb) || !extent(p.m, p.n, p.ldc, &ec))
        return fail(TG_ERR_INVALID_ARG, "matrix extent overflows int64");
    if (!p.unit()) {   // (rows-1)*rs + (cols-1)*cs + 1
        int64_t t1, t2;
        if (p.m > 0 && p.k > 0 && (mul_ovf(p.m - 1, p.lda, &t1) || mul_ovf(p.k - 1, p.csa, &t2) || add_ovf(t1, t2, &ea) || add_ovf(ea, 1, &ea)))
            return fail(TG_ERR_INVALID_ARG, "matrix extent overflows int64");
        if (p.k > 0 && p.n > 0 && (mul_ovf(p.k - 1, p.ldb, &t1) || mul_ovf(p.n - 1, p.csb, &t2) || add_ovf(t1, t2, &eb) || add_ovf(eb, 1, &eb)))
            return fail(TG_ERR_INVALID_ARG, "matrix extent overflows int64");
    }
    if (p.batch > 1) {
        if (p.strideC < ec) return fail(TG_ERR_INVALID_ARG, "strideC smaller than one output matrix");
        if (mul_ovf(p.batch - 1, p.strideA, &t) || add_ovf(t, ea, &t) || t > INT64_MAX / 4 ||
            mul_ovf(p.batch - 1, p.strideB, &t) || add_ovf(t, eb, &t) || t > INT64_MAX / 4 ||
            mul_ovf(p.batch - 1, p.strideC, &t) || add_ovf(t, ec, &t) || t > INT64_MAX / 4)
            return fail(TG_ERR_INVALID_ARG, "batch extent overflows int64");
    } else if (ea > INT64_MAX / 4 || eb > INT64_MAX / 4 || ec > INT64_MAX / 4) {
        return fail(TG_ERR_INVALID_ARG, "matrix extent overflows int64");
    }
    const bool out_nonempty = p.batch > 0 && p.m > 0 && p.n > 0;
    if (out_nonempty) {
        if (!p.C) return fail(TG_ERR_INVALID_ARG, "C is null");
        if (p.k > 0 && (!p.A || !p.B)) return fail(TG_ERR_INVALID_ARG, "A or B is null");
    }
    if (p.m > INT32_MAX || p.n > INT32_MAX || p.k > INT32_MAX || p.batch > INT32_MAX)
        return fail(TG_ERR_UNSUPPORTED, "a dimension exceeds 2^31-1");
    auto a16 = [](const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; };
    p.a_al = a16(p.A) && (p.batch <= 1 || p.strideA % 4 == 0);
    p.b_al = a16(p.B) && (p.batch <= 1 || p.strideB % 4 == 0);
    p.aligned = p.a_fits(0) && p.b_fits(0);
    return TG_OK;
}

tg_status check_device() {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(TG_ERR_HIP, std::string("hipGetDevice: ") + hipGetErrorString(e));
    if (dev < 0 || dev >= 64) return fail(TG_ERR_UNSUPPORTED, "device index out of range");
    std::lock_guard<std::mutex> lk(g_mutex);
    if (g_device_ok[dev] == 0) {
        hipDeviceProp_t prop;
        e = hipGetDeviceProperties(&prop, dev);
        if (e != hipSuccess) return fail(TG_ERR_HIP, std::string("hipGetDeviceProperties: ") + hipGetErrorString(e));
        g_device_ok[dev] = strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : -1;
    }
    if (g_device_ok[dev] < 0) return fail(TG_ERR_UNSUPPORTED, "the current device is not gfx950 (MI355X)");
    return TG_OK;
}

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Number of K ranges actually used when `want` are asked for, and K tiles per range.
void split_plan(const KernelInfo &ki, int64_t k, int want, int *splits, int *per) {
    const int64_t kt = std::max<int64_t>(ceil_div(k, ki.BK), 1);
    const int64_t pp = ceil_div(kt, std::max(want, 1));
    *per = (int)pp;
    *splits = (int)ceil_div(kt, pp);
}

// Packed copy of a rows x cols operand: rows padded to a multiple of 4 floats (16-byte rows).
int64_t pack_ld(int64_t cols) { return (cols + 3) / 4 * 4; }
size_t pack_bytes(int64_t rows, int64_t cols) { return (size_t)rows * (size_t)pack_ld(cols) * sizeof(float); }
// An operand is packed when more than one 128-wide tile row/column would fetch it.
constexpr int64_t kPackMinReuse = 128;

// Product of non-negative factors, saturating at INT64_MAX.
int64_t sat_mul(std::initializer_list<int64_t> f) {
    int64_t r = 1;
    for (int64_t x : f)
        if (mul_ovf(r, x, &r)) return INT64_MAX;
    return r;
}

int64_t sat_add(int64_t a, int64_t b) {
    int64_t r;
    return add_ovf(a, b, &r) ? INT64_MAX : r;
}

size_t ws_need(const Problem &p, int splits) {
    if (splits <= 1) return 0;
    const int64_t bytes = sat_mul({p.batch, (int64_t)splits, p.m, p.n, (int64_t)sizeof(float)});
    return bytes == INT64_MAX ? SIZE_MAX : (size_t)bytes;
}

// Bytes of the piece images a cut-ahead kernel writes (A's, then B's; every tile padded to full size).
size_t planes_need(const Problem &p, const KernelInfo &ki) {
    if (!ki.precut) return 0;
    const int64_t rows = sat_mul({ceil_div(p.m, ki.BM), (int64_t)ki.BM}), cols = sat_mul({ceil_div(p.n, ki.BN), (int64_t)ki.BN});
    if (rows == INT64_MAX || cols == INT64_MAX) return SIZE_MAX;
    const int64_t bytes = sat_mul({p.batch, ceil_div(p.k, ki.BK), rows + cols, (int64_t)(3 * (ki.BK / 8) * 16)});
    return bytes == INT64_MAX ? SIZE_MAX : (size_t)bytes;
}

// The two launches of a configuration with a tail split: rows [0, m1) with the configuration as it
// stands, rows [m1, m) with split-K tail_splits.  (Every problem of a batch is cut at the same row.)
void tail_parts(const Problem &p, const Config &c, Problem *p1, Config *c1, Problem *p2, Config *c2) {
    const KernelInfo &ki = tg::kernel(c.kernel);
    const int64_t m1 = (ceil_div(p.m, ki.BM) - c.tail) * ki.BM;
    *p1 = p;
    p1->m = m1;
    *p2 = p;
    p2->m = p.m - m1;
    if (p.A) p2->A = p.A + m1 * p.lda;
    if (p.C) p2->C = p.C + m1 * p.ldc;
    *c1 = c;
    c1->tail = 0;
    c1->tail_splits = 1;
    *c2 = *c1;
    c2->splits = c.tail_splits;
    // a tail range of at most kLongK terms does not need the second accumulator level: same tile without it
    if (ki.two_level) {
        int sp, per;
        split_plan(ki, p.k, c.tail_splits, &sp, &per);
        const std::string name = ki.name;
        const size_t at = name.find("_acc2");
        if ((int64_t)per * ki.BK <= kLongK && at != std::string::npos) {
            const int sib = find_kernel(name.substr(0, at) + name.substr(at + 5));
            if (sib >= 0) c2->kernel = sib;
        }
    }
}

// Workspace of a configuration: split-K partials (rounded up to 256 bytes), then the piece images.
size_t ws_total(const Problem &p, const Config &c) {
    if (c.tail > 0 && c.kernel >= 0 && c.tail < ceil_div(p.m, tg::kernel(c.kernel).BM)) {
        Problem p1, p2;
        Config c1, c2;
        tail_parts(p, c, &p1, &c1, &p2, &c2);
        return ws_total(p2, c2);
    }
    const size_t a = ws_need(p, c.splits), b = planes_need(p, tg::kernel(c.kernel));
    if (a == SIZE_MAX || b == SIZE_MAX || a > SIZE_MAX - 256 - b) return SIZE_MAX;
    return b == 0 ? a : (a + 255) / 256 * 256 + b;
}

// Row-panel variants that hold their rows of A in LDS for the whole K range (tile_resident_kernel.hpp).
bool resident_panel(const KernelInfo &ki) { return ki.name[0] == 'g' && strstr(ki.name, "_res_") != nullptr; }

// Is this configuration usable for this problem?  (static validity filter of the tuner:
// divisibility, alignment, accumulation depth, LDS capacity, workspace)
bool config_valid(const Problem &p, const Config &c, size_t ws_bytes, std::string *why = nullptr) {
    auto no = [&](const char *w) { if (why) *why = w; return false; };
    if (c.kernel < 0 || c.kernel >= tg::num_kernels()) return no("no such kernel");
    const KernelInfo &ki = tg::kernel(c.kernel);
    if (c.group < 1) return no("group must be >= 1");
    if (c.occ < 0 || c.occ > 16) return no("occupancy cap must be 0..16");
    if (c.persist < 0 || c.persist > 16) return no("persistent workgroups per CU must be 0..16");
    if ((c.persist > 0) != ki.persistent) return no("p<n> goes with the persistent kernel variants (names starting with p), and only with them");
    if (c.tail != 0) {
        if (c.tail < 0 || c.tail_splits < 2) return no("a tail split needs t<rows>x<splits> with rows >= 1 and splits >= 2");
        if (ki.kind != tg::KIND_TILE || ki.persistent || ki.precut) return no("no tail split for this kernel");
        if (c.splits != 1) return no("a tail split goes with s1");
        if (c.tail >= ceil_div(p.m, ki.BM)) return no("the tail must leave at least one tile row");
        Problem p1, p2;
        Config c1, c2;
        tail_parts(p, c, &p1, &c1, &p2, &c2);
        return config_valid(p1, c1, ws_bytes, why) && config_valid(p2, c2, ws_bytes, why);
    }
    if (ki.kind == tg::KIND_WAVE) {
        if (!p.unit()) return no("the wave kernel needs unit element strides");
        if (!ki.edge && (!p.aligned || p.n % (ki.BN / 16) != 0))
            return no("the wide wave tiles need 16-byte aligned operands and n a multiple of their lane width");
        if (c.splits != 1) return no("the wave kernel has no split-K");
        const int kw = std::max(1, ki.kwaves);   // waves that share a tile, each with its part of K
        if (p.k > (int64_t)kWaveMaxK * kw) return no("k too long for the single-accumulator wave kernel");
        if (sat_mul({ceil_div(p.m, ki.BM), ceil_div(p.n, ki.BN), p.batch}) > (int64_t)(4 / kw) * INT32_MAX) return no("too many tiles");
        return true;
    }
    if (ki.lds_bytes > kLdsPerCU) return no("tile needs more LDS than a CU has");
    if (ki.precut) {
        // the cutting passes take any A and B, the product kernel any C
        if (ws_total(p, c) > ws_bytes) return no("workspace too small for the piece images");
        if (sat_mul({p.batch, ceil_div(p.k, ki.BK), std::max(ceil_div(p.m, ki.BM), ceil_div(p.n, ki.BN))}) > INT32_MAX)
            return no("too many workgroups");
    } else if (!ki.edge) {
        if (ki.amode == 0 && ki.bmode == 0) {
            if (!p.aligned) return no("operands are not 16-byte aligned");
        } else if (!p.a_fits(ki.amode) || !p.b_fits(ki.bmode)) {
            return no("the operands do not lie as this variant reads them (plain / transposed with 16-byte aligned rows / strided)");
        }
        // K must fill whole tiles; ragged m and n are handled by re-reading the last row / vector
        // and masking the stores (the persistent variants walk exact tiles only)
        if (p.k % ki.BK && !(ki.k_tail && p.k % 4 == 0 && p.k >= ki.BK))
            return no(ki.k_tail ? "k is neither a multiple of the K tile nor (a multiple of 4 and at least one K tile)"
                                : "k is not a multiple of the K tile");
        if (ki.bmode == 0 && p.b_cols() % 4) return no("n is not a multiple of 4");
        if (ki.persistent && (p.m % ki.BM || p.n % ki.BN)) return no("sizes are not multiples of the tile");
        if (ki.persistent && ki.name[0] == 'g') {
            // a workgroup walks tiles / workgroups neighbouring column tiles of one row panel
            const int64_t tiles = (p.m / ki.BM) * (p.n / ki.BN), wgs = (int64_t)c.persist * kNumCUs;
            if (p.batch != 1 || c.splits != 1) return no("the walking row-panel variants take one problem and one K range");
            if (tiles % wgs || (p.n / ki.BN) % (tiles / wgs)) return no("the tiles of a row panel do not divide evenly over the workgroups");
            // (the variants that keep their rows of A in LDS over the whole K range: k + 8 floats per row, 64 KB per workgroup)
            if (resident_panel(ki) && (int64_t)ki.BM * (p.k + 8) * 4 > 64 * 1024)
                return no("the workgroup's rows of A over the whole K range do not fit its LDS");
        }
        if (ki.defer) {
            const int cb = ki.WN / 32;   // floats per store
            if (c.splits != 1) return no("this variant has no split-K");
            if ((reinterpret_cast<uintptr_t>(p.C) & (4 * cb - 1)) || p.ldc % cb || (p.batch > 1 && p.strideC % cb))
                return no("rows of C are not aligned for this variant's stores");
        }
        // the fast variants address inside a tile with 32-bit offsets
        {
            const int64_t span_a = ki.amode == 1 ? sat_add(sat_mul({ki.BK - 1, p.csa}), ki.BM)
                                                 : sat_add(sat_mul({ki.BM - 1, p.lda}), sat_mul({ki.BK, p.csa}));
            const int64_t span_b = ki.bmode == 1 ? sat_add(sat_mul({ki.BN - 1, p.csb}), ki.BK)
                                                 : sat_add(sat_mul({ki.BK - 1, p.ldb}), sat_mul({ki.BN, p.csb}));
            // (element offsets inside a tile are kept as 32-bit byte offsets)
            if (span_a >= (1 << 30) || span_b >= (1 << 30)) return no("leading dimension too large for the exact-fit kernels");
        }
        // (the rows of a lane's results are addressed with a 32-bit byte offset)
        if (p.ldc >= (1 << 27) || p.n >= (1 << 27)) return no("leading dimension of C too large for the exact-fit kernels");
        // (the bf16-piece kernels form 32-bit byte offsets)
        if (ki.pieces && ((ki.BM - 1) * p.lda + ki.BK >= (1 << 30) || (ki.BK - 1) * p.ldb + ki.BN >= (1 << 30)))
            return no("leading dimension too large for the exact-fit kernels");
    }
    int splits, per;
    split_plan(ki, p.k, c.splits, &splits, &per);
    if (splits != c.splits) return no("split count leaves an empty K range");
    const int64_t k_range = std::min<int64_t>((int64_t)per * ki.BK, p.k);
    if (ki.pieces ? k_range > kLongKPieces : (k_range > kLongK && !ki.two_level))
        return no("K range too long for a single accumulator level");
    if (c.splits > 1) {
        if (per < 2) return no("K range shorter than two tiles");
        if (ws_total(p, c) > ws_bytes) return no("workspace too small for this split");
    }
    const int64_t blocks = sat_mul({ceil_div(p.m, ki.BM), ceil_div(p.n, ki.BN), (int64_t)c.splits, p.batch});
    if (blocks > INT32_MAX) return no("too many workgroups");
    return true;
}

// Lower bound on the run time of a configuration (seconds): no kernel can beat the chip's
// MFMA peak, a wave cannot beat the one SIMD it runs on, workgroups cannot use more CUs
// than exist, and operands/results cross HBM at least once (Sec. 5.1 of the paper prunes
// candidates with such a bound; this is the flat-set version of that cut).
double lower_bound_seconds(const Problem &p, const Config &c) {
    if (c.tail > 0) {   // two launches, one after the other
        Problem p1, p2;
        Config c1, c2;
        tail_parts(p, c, &p1, &c1, &p2, &c2);
        return lower_bound_seconds(p1, c1) + lower_bound_seconds(p2, c2);
    }
    const KernelInfo &ki = tg::kernel(c.kernel);
    const double flops = 2.0 * p.batch * p.m * p.n * p.k;
    // the bf16 pipe multiplies 16x as fast as the fp32 one, and a piece kernel needs `pieces` products per product
    const double speed = ki.pieces ? 16.0 / ki.pieces : 1.0;
    double t = flops / (kPeakFlops * speed);
    int splits = 1, per = 1;
    int waves_per_block = ki.threads / 64;
    if (ki.name[0] == 'g') waves_per_block = (ki.BM / ki.WM) * (ki.BN / ki.WN);   // row-panel kernels: the other waves only gather
    double wave_flops;
    int64_t blocks;
    if (ki.kind == tg::KIND_WAVE) {
        const int kw = std::max(1, ki.kwaves);
        wave_flops = 2.0 * ki.BM * ki.BN * (double)ceil_div(p.k, kw);
        blocks = ceil_div(sat_mul({ceil_div(p.m, ki.BM), ceil_div(p.n, ki.BN), p.batch, (int64_t)kw}), 4);
    } else {
        split_plan(ki, p.k, c.splits, &splits, &per);
        // variants with several wave groups along K give every wave only its share of the K range
        const int kgroups = std::max(1, ki.threads / ((ki.BM / ki.WM) * (ki.BN / ki.WN) * 64));
        wave_flops = 2.0 * ki.WM * ki.WN * std::min<int64_t>((int64_t)per * ki.BK, p.k) / kgroups;
        blocks = ceil_div(p.m, ki.BM) * ceil_div(p.n, ki.BN) * splits * p.batch;
    }
    t = std::max(t, wave_flops / (kSimdFlops * speed));
    // workgroups are spread over at most kNumCUs CUs; each CU has 4 SIMDs
    const double rounds = (double)ceil_div(blocks * waves_per_block, (int64_t)kNumCUs * 4);
    t = std::max(t, rounds * wave_flops / (kSimdFlops * speed));
    double bytes = 4.0 * p.batch * ((double)p.m * p.k + (double)p.k * p.n + (double)p.m * p.n);
    if (splits > 1) bytes += 2.0 * 4.0 * p.batch * splits * (double)p.m * p.n;
    t = std::max(t, bytes / kPeakHbm);
    // kernels that cut ahead first stream both operands through two passes of their own (4 bytes in, 6 out)
    if (ki.precut) t += 10.0 * p.batch * ((double)p.m * p.k + (double)p.k * p.n) / kPeakHbm;
    return t;
}

// Rough cost model used only to rank candidates and as the fallback when nothing is tuned.
// A CU delivers its MFMA rate once it holds four waves; workgroups beyond one per CU queue up.
double heuristic_seconds(const Problem &p, const Config &c) {
    if (c.tail > 0) {   // the second launch follows the first without a host round trip
        Problem p1, p2;
        Config c1, c2;
        tail_parts(p, c, &p1, &c1, &p2, &c2);
        return heuristic_seconds(p1, c1) + heuristic_seconds(p2, c2) - 2e-6;
    }
    const KernelInfo &ki = tg::kernel(c.kernel);
    const double launch = 4e-6;
    if (ki.kind == tg::KIND_WAVE) {
        const int kw = std::max(1, ki.kwaves);
        const double waves = (double)ceil_div(p.m, ki.BM) * ceil_div(p.n, ki.BN) * p.batch * kw;
        const double per_simd = std::ceil(waves / (kNumCUs * 4.0));
        const double wave_flops = 2.0 * ki.BM * ki.BN * (double)ceil_div(p.k, kw);
        // a lone wave reads its operands with the latency exposed: one round trip per 64 k (32x32 tiles: half
        // the SIMD rate, 64x64x2048 in 49 us) or per 128 k (16x16 tiles: a third, the same product in 20.6 us);
        // several waves on one SIMD overlap, up to about a third of the rate (measured)
        // (waves that split K share nothing in L1 and overlap a little worse: 0.24 measured at 2000x100x500)
        double t = std::max(wave_flops / (kSimdFlops * (ki.BM == 32 ? 0.5 : 0.33)), per_simd * wave_flops / (kSimdFlops * (kw > 1 ? 0.24 : 0.3)));
        // the result leaves in rows of one tile width: 64-byte pieces from 16x16 tiles, full lines from 32x32
        // (2048x2048x32: 16 MB of C in 10 us and 7.2 us)
        t = std::max(t, 4.0 * p.batch * (double)p.m * p.n / (ki.BN <= 16 ? 1.6e12 : 2.3e12));
        // every tile fetches its own operands: L2 delivers about 10 TB/s (512^3 with 16x16 tiles: 6.4 us measured).
        // The four waves of a workgroup are neighbouring tiles of one tile row and share its A rows in L1, unless
        // they split K among themselves.
        const double a_share = kw > 1 ? 1.0 : 4.0;
        t = std::max(t, 4.0 * p.batch * (double)p.m * p.n * p.k * (1.0 / (ki.BM * a_share) + 1.0 / ki.BN) / 10e12);
        return launch + t + (kw > 1 ? 0.3e-6 : 0.0);   // the partial tiles meet in LDS behind a barrier
    }
    int splits, per;
    split_plan(ki, p.k, c.splits, &splits, &per);
    const double blocks = (double)ceil_div(p.m, ki.BM) * ceil_div(p.n, ki.BN) * splits * p.batch;
    const double per_cu = std::ceil(blocks / kNumCUs);
    if (ki.name[0] == 'g') {
        // Row panels of a gathered A (tile_panel_kernel.hpp).  Measured on MI355X: lines that miss L2 arrive at about
        // 5e10 lines/s over the whole chip and 2.4e8 per CU (an element asked for again by another column tile costs
        // about a third of that), B streams through a CU at about 125 GB/s beside the gather and is hidden while the
        // CU's own request rate is the limit; the 16x16x4 products run at 93 % of the MFMA rate (1024^3 at stride 2:
        // 21 us in all); a K range of few chunks pays its pipeline fill; a K split pays the partial products' way out and back.
        // (us, A at element stride 32, 16x1024 / 16x512 / 32x512 / 32x1024 panels: 1024^3 s2 51 38 52 79, s4 43 40 42 56;
        // 2048^3 s1 224 244 229 -, s2 238 249 246 200; 4096x1024x1024 s1 148 141 134 188; 4096x4096x1024 s1 395 425 438 342;
        // 8192x512x1024 s1 238 210 187 222; stride 8, 1024^3: s2 40 28 41 69)
        const double k_range = (double)std::min<int64_t>((int64_t)per * ki.BK, p.k);
        const double line = std::min(4.0 * p.csa, 128.0);
        if (ki.persistent && (resident_panel(ki) || (p.a_class() == 0 && p.k <= 448))) {
            // Short K, one walk per workgroup.  A resident in LDS (tile_resident_kernel.hpp): the panel is gathered once per
            // workgroup, in front of the products and not beside them; from there the waves run at 96.5 % of the MFMA rate
            // and what shows of C's way out is a twentieth of a microsecond per MB (us, plain operands, measured / this
            // model: 4096x4096x64 22.1 / 22.0, x128 36.0 / 36.7, x256 64.2 / 66, x448 108.5 / 110; 8192x8192x128 137 / 132;
            // 2048x2048x128 12.4 / 12.7; 8192x4096x192 98 / 97).  The walking panels that re-gather A per tile behind a
            // barrier per chunk are about a microsecond behind on the same shapes (4096x4096x128 37.2, x64 22.8, x256 65.7)
            // and, from k = 512 on, no longer ahead of the tile kernels (4096x4096x512 123 - 126 against 123).
            // (the workgroups of one row panel run on one XCD: the first to ask for a line of A brings it into their L2, the
            // others find it there at about eight times the rate.  A at stride 32, time of the gather alone, us measured /
            // this model: 4096x4096x128, two workgroups per panel 8.4 / 9.6; 4096x4096x320, two 21 / 24; 2048x4096x384,
            // four 13 / 17)
            const double wgs = std::max(1, c.persist) * (double)kNumCUs;
            const double wgs_per_row = std::max(1.0, wgs / (double)ceil_div(p.m, ki.BM));
            const double per_el = std::max(line / 128.0, line >= 32.0 ? 0.5 : (line >= 16.0 ? 0.35 : 0.25));
            const double miss_share = line / 128.0;
            const double req = ki.BM * (double)p.k * per_el * (1.0 + (wgs_per_row - 1.0) / 8.0) / wgs_per_row;
            const double t_cu = std::max(1, c.persist) * req * (miss_share + (1.0 - miss_share) / 3.0) / 2.4e8;
            const double t_chip = (double)p.m * p.k * line / 128.0 / 5e10;
            const double t_mfma = 2.0 * (double)p.m * p.n * p.k / (kNumCUs * 4.0 * kSimdFlops * 0.965);
            double t = launch + std::max(t_chip, t_cu) + t_mfma + 4.0 * (double)p.m * p.n / 20e12;
            // (few rows: hardly anybody has fetched a line of B before the wave that needs it, and one or three steps of
            // prefetch do not cover a miss.  256x16384x256 22.9 us on 32-row and 26.9 us on 16-row panels against 20.1 us
            // on 64x64 tiles, 256x8192x448 21.5 against 17.0 us; from 512 rows on the panels are level or ahead:
            // 512x16384x128 21.4 against 23.8 us, 512x8192x256 18.9 against 19.9 us)
            if (p.m < 512) t *= 1.25;
            if (!resident_panel(ki)) t = (t + 1.0e-6) * (ki.two_level ? 1.01 : 1.0) + (strstr(ki.name, "_b3") ? 0.3e-6 : 0.0);
            else t = t * (ki.threads < 1024 ? 1.0 : 1.005) + (strstr(ki.name, "_b3") ? 0.1e-6 : 0.0);
            // (sixteen waves in one workgroup: on a par on most shapes, 8192x8192x64 97 us against 82 us; three steps of B
            // ahead: within 2 % either way)
            return t;
        }
        const double per_el = std::max(line / 128.0, line >= 32.0 ? 0.5 : (line >= 16.0 ? 0.35 : 0.25));
        const double tiles_n = (double)ceil_div(p.n, ki.BN);
        const double miss_share = line / 128.0;          // share of the requests that bring a new line
        const double req = ki.BM * k_range * per_el * (1.0 + (tiles_n - 1.0) / 3.0) / tiles_n;
        // (the 2.4e8 requests/s of a CU were measured with all 256 CUs gathering, where they are the chip's line rate
        // seen from one CU; with fewer workgroups than CUs each gets more of it, up to about 6.5e8: 1024x256x1024 at
        // stride 32, 64 workgroups of 16384 lines each, 31.6 us in all)
        const double active = std::min(blocks, (double)kNumCUs);
        const double cu_rate = std::min(6.5e8, 1.25 * 5e10 / std::max(active, 1.0));
        const double t_cu = per_cu * req * (miss_share + (1.0 - miss_share) / 3.0) / cu_rate;
        // (a workgroup that walks several tiles of its row panel gathers the panel again for each of them, one after the
        // other: at a large stride the lines have left L2 by then and cross the fabric once per tile, where the tiles of
        // one-tile workgroups run side by side and share them.  us, A at stride 32, walking / one tile per workgroup:
        // 4096x4096x128 95 / 61, 2048x2048x256 52 / 26, 4096x4096x320 205 / 113; at stride 2 - 8 the walk wins: 38 / 45)
        const double walked = ki.persistent && c.persist > 0 ? std::max(1.0, blocks / ((double)c.persist * kNumCUs)) : 1.0;
        const double t_chip = p.batch * (double)p.m * p.k * line / 128.0 / 5e10 * (1.0 + (walked - 1.0) * line / 128.0);
        const double t_b = per_cu * k_range * (double)std::min<int64_t>(ki.BN, p.n) * 4.0 / 1.25e11;
        const double t_gather = std::max(t_chip, t_cu);
        const double t_mem = std::max(t_chip + 0.8 * t_b, t_cu);      // B's line requests take slots from the gather
        // (64-column wave tiles: twice the compute waves per SIMD, 2 - 5 % ahead of 128-column ones on every shape swept)
        const double t_mfma = per_cu * 2.0 * ki.BM * ki.BN * k_range / (4.0 * kSimdFlops * (ki.WN == 64 ? 0.95 : 0.93));
        const double t_comp = std::max(t_mfma, t_b);                  // B is fetched by the compute waves, behind their MFMAs
        // (B fetched three steps ahead instead of one: the compute waves stall less on it, reach the barrier sooner, and
        // the producers wait less for free stages: stride 32, us: 1024^3 on 16x256 panels 37.3 -> 33.0, 4096x1024x1024 on
        // 32x512 panels 127 -> 122, 2048^3 224 -> 210, 1024^3 at stride 8 28 -> 21.6; two chunks of pipeline fill instead of one:
        // 4096x4096x128 44 -> 48)
        const bool deep_b = strstr(ki.name, "_b3") != nullptr;
        // (a workgroup that walks several tiles of its row panel fills its pipeline once for all of them)
        // (where the gather is the longer part the fill is mostly gather that has to happen anyway: 1024x1024x256 at
        // stride 32 11.4 us where a full charge for two chunks said 17.4)
        const double fill = 1.0 + (t_mem >= t_comp ? 0.25 : 1.0) * (deep_b ? 2.0 : 1.0) * ki.BK / (k_range * walked);
        // (what shows of the shorter part: half of the gather where the products are longer; where the gather is, 15 % of
        // the products when they are far shorter and up to 70 % near parity, where the two roles keep waiting for each other)
        double body;
        if (t_mem >= t_comp) {
            const double l = std::log(t_comp / std::max(t_mem, 1e-9));
            body = t_mem + (0.15 + 0.55 * std::exp(-l * l / (2.0 * 0.35 * 0.35))) * t_comp;
        } else {
            body = t_comp + 0.5 * t_gather + 0.25 * std::max(0.0, t_mem - t_gather);
        }
        double t = launch + 1e-6 + body * fill * (deep_b ? 0.9 : 1.0);
        if (p.a_class() == 0) {
            // Plain operands.  Where the 32 x 512 panels fill every CU the same number of times and K is long, the deep
            // chunks run at 96 % of the MFMA rate plus 3.3 us per round of workgroups, which no tile kernel reaches (us, these
            // panels / the tile kernel chosen before: 2048^3 119.5 / 123, 2048x2048x8192 463 / 499, 4096x4096x2048 469 / 474,
            // 4096x4096x8192 1837 / 1858, 6144^3 3089 / 3132, 8192^3 7277 / 7348, 1024x4096x2048 120 / 126); with a
            // partial last round they lose by as much as that round is empty (3072^3 518 / 407, 2048x1024x4096 230 / 126),
            // and on batches the tile kernels are level or 1 % ahead (64 of 512x512x2048: 503 / 497).
            // Elsewhere they stay behind the tile kernels until the tuner has timed both.
            const int64_t blocks_i = ceil_div(p.m, ki.BM) * ceil_div(p.n, ki.BN) * p.batch;
            if (deep_b && ki.BK >= 128 && ki.BM == 32 && p.b_class() == 0 && p.batch == 1 && splits == 1 && p.k >= 2048 && p.m % ki.BM == 0 &&
                p.n % ki.BN == 0 && blocks_i % kNumCUs == 0)
                return launch + (double)(blocks_i / kNumCUs) * 3.25e-6 +
                       2.0 * p.batch * (double)p.m * p.n * p.k / (kPeakFlops * (ki.BK >= 256 ? 0.961 : 0.959));
            t *= 1.15;
        }
        if (splits > 1) t += 2.5e-6 + 4.0 * p.batch * (2.0 * splits + 1.0) * (double)p.m * p.n / 5e12;
        return t;
    }
    // operand traffic per flop falls with the wave tile; predication and the second
    // accumulator level cost a little
    // (measured on MI355X: K tiles of 32 beat 16 by ~1 %, direct-to-LDS loads win by ~1 % on
    // the large tiles, persistent variants only pay for short K; element-strided operands
    // cost the predicated kernels another factor of about two)
    // (constants refitted after the K loops lost a third of their non-MFMA instructions: the register-staged kernels
    // gained most, small wave tiles lost less to large ones than before; sweep of 24 shapes, first choice against the
    // best of the model's ten first)
    double eff = 1.0 / (1.0 + 6.0 / ki.WM + 6.0 / ki.WN) * (ki.edge ? 0.75 : 1.0) * (ki.two_level ? 0.97 : 1.0);
    eff *= ki.BK >= 32 ? 1.0 : 0.985;
    // (direct-to-LDS loads: 2 % behind the register-staged kernels on the large tiles, ahead on 64x64 tiles with
    // k >= 256, behind on 128x128; the 128x128 wave tile, 256 accumulator registers, a further 7 % behind)
    if (ki.name[0] == 'd') eff *= ki.WM * ki.WN > 64 * 64 ? (ki.WM * ki.WN >= 128 * 128 ? 0.92 : 0.985) : (ki.WM * ki.WN == 32 * 32 ? 1.04 : 0.97);
    // two workgroups resident per CU cover each other's barrier and load waits (4096^3 on 128x128 tiles with a second
    // accumulator level: 94 % of the MFMA rate, against 86 % at 2048^3 where every CU holds one)
    if (ki.kind == tg::KIND_TILE && !ki.persistent && 2 * ki.lds_bytes <= kLdsPerCU && ki.WM * ki.WN <= 64 * 64 && blocks >= 2.0 * kNumCUs)
        eff *= 1.05;
    // (32x32 wave tiles with the fragments of a whole K tile fetched one tile ahead: 1024^3 20.0 us against 21.7 us;
    // K tiles of 64 in that form: 21.0 us)
    if (strstr(ki.name, "_tf")) eff *= ki.BK > 32 ? 1.03 : 1.08;
    if (ki.name[0] == 'd') {
        // deeper rings and wave groups along K are there for the tuner to try; untuned, the plain form goes first
        // (a ring deeper than the K range only adds loads: 1536x1536x64 11.3 us against 9.2 us)
        const int stages = ki.lds_bytes / ((ki.BM * ki.BK + ki.BK * ki.BN) * 4);
        if (stages > 2) eff *= p.k < 8 * ki.BK ? 0.85 : 0.995;
        if (ki.threads > (ki.BM / ki.WM) * (ki.BN / ki.WN) * 64) eff *= 0.97;
    }
    // the 32-wide and 32-tall tiles are for skinny products; on others they re-fetch the long operand too often
    if ((ki.BN <= 32 && p.n > 32) || (ki.BM <= 32 && p.m > 32)) eff *= 0.9;
    if (ki.persistent) eff *= p.k <= 256 ? 1.0 : 0.95;
    if (!p.unit() && ki.edge) eff *= 0.5;
    // (wave tiles of 16 rows on the 16x16x4 instruction: 1024^3 with plain operands 35 us against 27 us for 32x128 tiles)
    if (ki.WM < 32) eff *= 0.8;
    // transposed operands read as they lie cost a few more LDS reads per MFMA
    if (ki.amode == 1) eff *= 0.985;
    if (ki.bmode == 1) eff *= 0.985;
    // a tile of which at most a quarter is real output (tiny problems of a batch): the waves
    // that hold only padding still take their share of the loads, the barrier and the MFMA pipe
    if (p.m * 2 <= ki.BM && p.n * 2 <= ki.BN) eff *= 0.8;
    const double block_flops = 2.0 * ki.BM * ki.BN * std::min<int64_t>((int64_t)per * ki.BK, p.k);
    // bf16-piece kernels: 16/pieces times the multiply rate; measured at 4096^3 they deliver 53 % of that
    // (cutting in the loop) and 59 % (cut ahead): the bf16 pipe runs at 1.8 GHz under load, not 2.4
    // (the in-loop cut costs vector instructions in proportion to BM + BN per BM * BN of products: smaller tiles
    // pay more; measured 0.53 / 0.45 / 0.36 of the bf16 rate for 128x256 / 128x128 / 64x64)
    if (ki.pieces) {
        const double tile = ki.precut ? 1.0 : std::min(1.0, 0.55 + 0.45 * ((double)ki.BM * ki.BN / (ki.BM + ki.BN)) / (128.0 * 256 / 384));
        eff = (ki.precut ? 0.59 : 0.53) * tile * 16.0 / ki.pieces;
    }
    const double cu_rate = std::min(ki.threads / 64, 4) * kSimdFlops * eff;
    // 1 us: the first K tile's trip through LDS and the epilogue, which the wave kernels do not have (a sweep of
    // 30 small and mid-size shapes: the model's first choice then averages 5 % above the best measured candidate)
    // (the first K tile of a workgroup is fetched and staged before anything is multiplied: half a tile's worth of its
    // time shows on short K ranges, 4096x4096x128 with K tiles of 32 43 us against 40 us with tiles of 16)
    const double fill = 1.0 + 0.5 * ki.BK / (double)std::min<int64_t>((int64_t)per * ki.BK, p.k);
    double t = launch + 1e-6 + per_cu * block_flops / cu_rate * fill;
    // A gathered operand: every element costs a line request (its own cache line when the stride is large) in every tile
    // that fetches it.  Measured with hardware counters on 1024^3 with A at element stride 32: a CU's L1 keeps about a
    // hundred line requests in flight at 450 cycles (L2 hit) to 1400 cycles (miss) each, which comes to 1.1 - 1.5 ns
    // per request and CU, and the distinct lines arrive from the fabric on top of that unless every workgroup is
    // resident at once on tiles of few rows, where the two overlap for the most part.  Constants from sweeps of all
    // gathering variants (us, stride 32: 1024^3 16x256 45, 32x128 51, 64x64 77, 128x128 162; 2048^3 431, 409, 794, 543;
    // 4096x1024x1024 227, 229, 418, 288; 1024x4096x1024 167, 173, 269, 183; stride 16, 1536^3: 144, 125, 178, 179;
    // stride 4, 3072^3: 674, 542, 605, 644).
    if (ki.amode == 2 || ki.bmode == 2) {
        const double line_a = std::min(4.0 * p.csa, 128.0), line_b = std::min(4.0 * p.csb, 128.0);
        // line requests per element of a gathered operand: neighbours in one line share a request, down to a floor
        // that the 4-byte loads themselves set (a quarter of a wave per cycle whatever the addresses)
        auto per_element = [](double line) { return std::max(line / 128.0, line >= 32.0 ? 0.5 : (line >= 16.0 ? 0.35 : 0.25)); };
        // line requests of one workgroup: per element of a gathered operand, per 128 bytes of a plain one
        const double req_a = ki.amode == 2 ? (double)ki.BM * p.k * per_element(line_a) : (double)ki.BM * p.k / 32.0;
        const double req_b = ki.bmode == 2 ? (double)ki.BN * p.k * per_element(line_b) : (double)ki.BN * p.k / 32.0;
        double lines = 0;
        if (ki.amode == 2) lines += p.batch * (double)p.m * p.k * line_a;
        if (ki.bmode == 2) lines += p.batch * (double)p.k * p.n * line_b;
        // tiles of few rows of a gathered A (and a plain B): more requests in flight per line of output, and their
        // misses stream at nearly the memory rate
        const bool few_rows = ki.amode == 2 && ki.bmode != 2 && ki.BM <= 32;
        const double per_req = few_rows ? (ki.BM <= 16 ? 1.5e-9 : 1.15e-9) : 1.12e-9;
        const double t_req = per_cu * (req_a + req_b) / splits * per_req, t_lines = lines / (few_rows ? 6e12 : 3.2e12);
        const bool overlapped = per_cu <= 1 && few_rows;
        const double t_gather = launch + 1e-6 + (overlapped ? std::max(t_req, t_lines) + 0.25 * std::min(t_req, t_lines) : t_req + t_lines);
        // (over several rounds the waits of the gather and the products overlap only in part: 4096^3 at stride 8 with
        // 128x256 tiles takes 1350 us where the product alone takes 975 us)
        t = std::max(t, t_gather) + (overlapped ? 0.0 : 0.35 * std::min(t, t_gather));
    }
    if (splits > 1) t += 4e-6 + 2.0 * 4.0 * p.batch * splits * (double)p.m * p.n / (kPeakHbm * 0.5);
    if (ki.precut) t += 6e-6 + 10.0 * p.batch * ((double)p.m * p.k + (double)p.k * p.n) / (kPeakHbm * 0.6);
    return t;
}

std::vector<Config> candidates(const Problem &p, size_t ws_bytes) {
    std::vector<Config> out;
    static const int kSplits[] = {1, 2, 3, 4, 6, 8, 12, 16};
    for (int ki = 0; ki < tg::num_kernels(); ++ki) {
        for (int s : kSplits) {
            Config c;
            c.kernel = ki;
            c.splits = s;
            c.group = kDefaultGroup;
            c.persist = tg::kernel(ki).persistent ? (tg::kernel(ki).name[0] == 'g' ? 1 : 2) : 0;   // workgroups per CU
            if (!config_valid(p, c, ws_bytes)) continue;
            const KernelInfo &kinfo = tg::kernel(ki);
            if (kinfo.pieces && g_math != TG_MATH_BF16_PIECES) continue;   // only on request
            // a variant that gathers or reads a transposed operand is offered for operands that lie that way (it is
            // valid, and can be forced, for anything it can read: a gather takes plain rows too, only slower)
            // (the row-panel kernels are also offered on plain operands, which their 4-byte gather reads as well: measured
            // on a par with the tile kernels on mid-size products and up to 5 % ahead, 2048^3 120 us against 127 us; the
            // cost model keeps them behind untuned, the tuner times them.  Only the forms with B three steps ahead,
            // and only where K is long enough for their pipeline)
            // (... or, for a short K, the forms in which a workgroup walks along its row panel: 4096x4096x128 37.2 us
            // against 38.7 us for the best tile kernel)
            const bool panel_on_plain = kinfo.name[0] == 'g' && p.a_class() == 0 && p.b_class() == 0 && p.aligned && s == 1 &&
                                        (kinfo.persistent ? p.k <= 512 : (strstr(kinfo.name, "_b3") && p.k >= 512));
            if (!panel_on_plain && (kinfo.amode || kinfo.bmode) && (kinfo.amode != p.a_class() || kinfo.bmode != p.b_class())) continue;
            if (kinfo.amode == 2) c.group = 1;            // a gathered A: the tiles that share a row panel of A run side by side
            else if (kinfo.bmode == 2) c.group = 64;      // a gathered B: those that share a column panel of B
            if (kinfo.kind == tg::KIND_TILE && kinfo.two_level && kinfo.amode == 0 && kinfo.bmode == 0) {
                // second-level accumulators only cost registers when the K range is short
                int sp, per;
                split_plan(kinfo, p.k, s, &sp, &per);
                if (std::min<int64_t>((int64_t)per * kinfo.BK, p.k) <= kLongK) continue;
            }
            // splitting only pays while the chip is under-filled
            if (s > 1) {
                const KernelInfo &k = tg::kernel(ki);
                const int64_t base = ceil_div(p.m, k.BM) * ceil_div(p.n, k.BN) * p.batch;
                if (base >= kNumCUs || base * s > 4 * kNumCUs) continue;
            }
            out.push_back(c);
        }
    }
    // Tail splits: when the tile count is a little above a multiple of what the chip holds at once, the
    // last round would run nearly empty; its tile rows go out as a second launch, split along K so that
    // they fill the chip once more for a fraction of a round.
    {
        const size_t n_plain = out.size();
        for (size_t i = 0; i < n_plain; ++i) {
            const Config base = out[i];
            const KernelInfo &k = tg::kernel(base.kernel);
            if (k.kind != tg::KIND_TILE || k.persistent || k.precut || base.splits != 1) continue;
            // (every problem of a batch is cut at the same tile row: a tile row of the batch is batch * tn tiles)
            const int64_t tm = ceil_div(p.m, k.BM), tn = ceil_div(p.n, k.BN) * p.batch, tiles = tm * tn;
            for (int per_cu = 1; per_cu <= 2; ++per_cu) {
                if (per_cu * k.lds_bytes > kLdsPerCU) break;
                const int64_t slots = (int64_t)kNumCUs * per_cu;
                const int64_t rest = tiles % slots;
                if (tiles <= slots || rest == 0) continue;
                const int64_t rows = ceil_div(rest, tn);
                if (rows >= tm) continue;
                // the K split of the tail: the two that the cost model likes best, if it likes them better
                // than the single launch (a tail of more than half a round can still gain: 140 tiles split
                // 3 ways are 2 rounds of a third of K)
                const double plain = heuristic_seconds(p, base);
                std::vector<std::pair<double, Config>> ranked;
                for (int sp : kSplits) {
                    if (sp < 2) continue;
                    Config h = base;
                    h.tail = (int)rows;
                    h.tail_splits = sp;
                    if (!config_valid(p, h, ws_bytes)) continue;
                    const double t = heuristic_seconds(p, h);
                    if (t < plain) ranked.emplace_back(t, h);
                }
                std::sort(ranked.begin(), ranked.end(), [](const std::pair<double, Config> &a, const std::pair<double, Config> &b) { return a.first < b.first; });
                for (size_t r = 0; r < ranked.size() && r < 2; ++r) out.push_back(ranked[r].second);
            }
        }
    }
    // an edge kernel is only interesting when no exact-fit kernel exists
    bool have_exact = false;
    for (const Config &c : out)
        if (tg::kernel(c.kernel).kind == tg::KIND_TILE && !tg::kernel(c.kernel).edge) have_exact = true;
    if (have_exact) {
        out.erase(std::remove_if(out.begin(), out.end(), [](const Config &c) {
                      return tg::kernel(c.kernel).kind == tg::KIND_TILE && tg::kernel(c.kernel).edge; }),
                  out.end());
    }
    std::sort(out.begin(), out.end(), [&](const Config &a, const Config &b) {
        return heuristic_seconds(p, a) < heuristic_seconds(p, b);
    });
    return out;
}

// Shape class of a problem: operand layout (0 unit strides off the 16-byte grid, 1 aligned, 2 + 3 * class of A + class of B
// for transposed / element-strided operands: 0 plain, 1 transposed and aligned, 2 anything else) + 16 x math mode.
ShapeKey key_of(const Problem &p) {
    const int layout = p.aligned ? 1 : (p.unit() ? 0 : 2 + 3 * p.a_class() + p.b_class());
    return ShapeKey(p.batch, p.m, p.n, p.k, layout + 16 * g_math);
}

// Element strides of gathered operands by the share of a cache line that an element costs: 0 not gathered or
// unit stride, then strides 2, 3-4, 5-8, 9-16, 17 and more (a line per element).  8 x A's + B's.
int stride_signature(const Problem &p) {
    auto bucket = [](int64_t cs) {
        int b = 0;
        while (b < 5 && (int64_t(1) << b) < cs) ++b;
        return b;
    };
    return 8 * (p.a_class() == 2 ? bucket(p.csa) : 0) + (p.b_class() == 2 ? bucket(p.csb) : 0);
}

// forced > tuned > heuristic.  Caller holds g_mutex.
tg_status choose(const Problem &p, size_t ws_bytes, Config *out) {
    read_env_once();
    if (g_forced) {
        std::string why;
        if (!config_valid(p, g_force_cfg, ws_bytes, &why)) {
            const bool ws_issue = ws_total(p, g_force_cfg) > ws_bytes;
            return fail(ws_issue ? TG_ERR_WORKSPACE : TG_ERR_INVALID_ARG,
                        "forced configuration " + spec_of(g_force_cfg) + " is not valid here: " + why);
        }
        *out = g_force_cfg;
        return TG_OK;
    }
    auto it = g_cache.find(key_of(p));
    if (it != g_cache.end() && config_valid(p, it->second.cfg, ws_bytes) &&
        (g_math == TG_MATH_BF16_PIECES || !tg::kernel(it->second.cfg.kernel).pieces)) {
        *out = it->second.cfg;
        return TG_OK;
    }
    // Ranking the candidates costs some 10 us; the outcome depends only on the shape class and on
    // the workspace size, so it is kept (a call must not spend longer choosing than launching).
    // (for a gathered operand the ranking also depends on how far apart its elements lie)
    ShapeKey shape = key_of(p);
    std::get<4>(shape) += 256 * stride_signature(p);
    const auto hkey = std::make_pair(shape, ws_bytes);
    auto hit = g_heuristic_choice.find(hkey);
    if (hit != g_heuristic_choice.end() && config_valid(p, hit->second, ws_bytes)) {
        *out = hit->second;
        return TG_OK;
    }
    std::vector<Config> cands = candidates(p, ws_bytes);
    if (cands.empty()) return fail(TG_ERR_INTERNAL, "no kernel variant is valid for this problem");
    *out = cands.front();
    if (g_heuristic_choice.size() >= 4096) g_heuristic_choice.clear();
    g_heuristic_choice[hkey] = *out;
    return TG_OK;
}

// 2-D split of the tile grid over the 8 XCDs: among the factorisations xm * xn == 8 that
// divide the grid, take the one whose regions touch the fewest operand elements
// (region rows + region columns); none fits -> linear ranges (xcd_m = xcd_n = 0).
void choose_xcd_split(const KernelInfo &ki, const Problem &p, GemmParams &g) {
    g.xcd_m = g.xcd_n = 0;
    if (ki.kind != tg::KIND_TILE) return;
    int64_t best = INT64_MAX;
    for (int xm = 1; xm <= 8; xm *= 2) {
        const int xn = 8 / xm;
        if (g.tiles_m % xm || g.tiles_n % xn) continue;
        // (an element of a gathered operand costs a whole cache line, or its share of one)
        const int64_t wa = ki.amode == 2 ? std::min<int64_t>(p.csa, 32) : 1, wb = ki.bmode == 2 ? std::min<int64_t>(p.csb, 32) : 1;
        const int64_t cost = (int64_t)(g.tiles_m / xm) * ki.BM * wa + (int64_t)(g.tiles_n / xn) * ki.BN * wb;
        if (cost < best) { best = cost; g.xcd_m = xm; g.xcd_n = xn; }
    }
}

tg_status launch(const Problem &p, const Config &c, void *ws, hipStream_t stream) {
    if (c.tail > 0) {
        Problem p1, p2;
        Config c1, c2;
        tail_parts(p, c, &p1, &c1, &p2, &c2);
        const tg_status st = launch(p1, c1, ws, stream);
        return st != TG_OK ? st : launch(p2, c2, ws, stream);
    }
    const KernelInfo &ki = tg::kernel(c.kernel);
    GemmParams g;
    memset(&g, 0, sizeof g);
    g.A = p.A; g.B = p.B; g.C = p.C;
    g.lda = p.lda; g.ldb = p.ldb; g.ldc = p.ldc;
    g.csa = p.csa; g.csb = p.csb;
    g.strideA = p.strideA; g.strideB = p.strideB; g.strideC = p.strideC;
    g.m = (int)p.m; g.n = (int)p.n; g.k = (int)p.k; g.batch = (int)p.batch;
    g.nb = (int)p.b_cols();
    g.tiles_m = (int)ceil_div(p.m, ki.BM);
    g.tiles_n = (int)ceil_div(p.n, ki.BN);
    g.group = std::min(c.group, g.tiles_m);
    choose_xcd_split(ki, p, g);
    g.splits = 1;
    g.ktiles_per_split = (int)std::max<int64_t>(ceil_div(p.k, ki.BK), 1);
    g.flush_tiles = ki.two_level ? std::max(1, kFlushK / ki.BK) : 0;
    g.max_blocks_per_cu = c.occ;
    g.persistent_blocks = c.persist > 0 ? c.persist * kNumCUs : 0;   // a multiple of 8
    g.flags = 0;
    {
        if (p.csa == 1) g.flags |= tg::kFlagVecA;
        if (p.csb == 1) g.flags |= tg::kFlagVecB;
        if (p.n % 4 == 0) g.flags |= tg::kFlagVecC;
    }
    if (ki.kind == tg::KIND_TILE && c.splits > 1) {
        split_plan(ki, p.k, c.splits, &g.splits, &g.ktiles_per_split);
        g.ws = static_cast<float *>(ws);
    }
    if (ki.precut) g.planes = static_cast<char *>(ws) + (ws_need(p, c.splits) + 255) / 256 * 256;
    hipError_t e = ki.launch(g, stream);
    if (e == hipSuccess && g.splits > 1) {
        e = tg::launch_splitk_reduce(g, stream);
    }
    if (e != hipSuccess)
        return fail(TG_ERR_HIP, std::string("launch of ") + ki.name + " failed: " + hipGetErrorString(e));
    return TG_OK;
}

tg_status zero_fill(const Problem &p, hipStream_t stream) {
    GemmParams g;
    memset(&g, 0, sizeof g);
    g.C = p.C; g.ldc = p.ldc; g.strideC = p.strideC;
    g.m = (int)p.m; g.n = (int)p.n; g.batch = (int)p.batch;
    hipError_t e = tg::launch_zero_fill(g, stream);
    if (e != hipSuccess) return fail(TG_ERR_HIP, std::string("zero fill failed: ") + hipGetErrorString(e));
    return TG_OK;
}

// Unit-stride operands that the exact-fit kernels cannot take as they are (a base or leading dimension off
// the 16-byte grid, k or n not a multiple of 4): when the product is large enough for it to pay and the
// workspace has room, A and/or B are copied once into aligned, zero-padded buffers at the front of the
// workspace and the product runs on the copies with k rounded up to a multiple of 4, or of 32 when both are copied
// and k >= 1000 (the padding is zero on both sides), and B fetched up to n rounded up.  C is written where it is (element stores if need be).
// Without room the predicated kernels take the operands as they are.  One problem only (no batches).
constexpr double kAlignMinWork = 4.2e8;   // m * n * k from which they pay
constexpr int64_t kAlignMinSize = 256;   // m and n from which the copies pay (a copy costs what one tile row's fetch does)
tg_status align_operands(Problem &p, void *&ws, size_t &ws_bytes, hipStream_t s, std::string *tag) {
    if (!p.unit() || p.batch != 1 || p.m < kAlignMinSize || p.n < kAlignMinSize || p.k < 32) return TG_OK;
    // below about 750^3 the wave kernels, which take any operands, beat two copy launches plus a tile kernel
    // (701^3: 17.8 us against 21.9 us with copies; 801^3: 39.9 us on the predicated tiles against 30.3 us)
    if ((double)p.m * p.n * p.k < kAlignMinWork) return TG_OK;
    // (in the piece mode, products of the size those kernels win at go to the ones that cut ahead, which take
    // the operands as they are: their cutting passes are the only copy needed)
    if (g_math == TG_MATH_BF16_PIECES && p.m * p.n >= (int64_t)1 << 20 && p.k >= 512) return TG_OK;
    auto a16 = [](const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; };
    const bool k_odd = p.k % 4 != 0, n_odd = p.n % 4 != 0;
    const bool copy_a = k_odd || !a16(p.A) || p.lda % 4 != 0;
    const bool copy_b = k_odd || n_odd || !a16(p.B) || p.ldb % 4 != 0;
    if (!copy_a && !copy_b) return TG_OK;
    // (with both operands copied anyway, K is padded to a whole K tile of 32 instead of a multiple of 4: the zeros cost
    // up to 3 % more products from k = 1000 on and open the problem to the direct-to-LDS kernels, which take whole
    // tiles only: 1025 x 1028 x 1028 36.3 us, x 1056 34.0 us; 2049 x 2052 x 2052 159 us, x 2080 152 us)
    const int64_t k4 = copy_a && copy_b && p.k >= 1000 ? ceil_div(p.k, 32) * 32 : pack_ld(p.k), n4 = pack_ld(p.n);
    const size_t need_a = copy_a ? (size_t)p.m * k4 * sizeof(float) : 0;
    const size_t need_b = copy_b ? (size_t)k4 * n4 * sizeof(float) : 0;
    if (need_a + need_b > ws_bytes || (reinterpret_cast<uintptr_t>(ws) & 15u) != 0) return TG_OK;
    char *w = static_cast<char *>(ws);
    hipError_t e = hipSuccess;
    if (copy_a && copy_b)       // one launch for both
        e = tg::launch_pad_copy2(p.A, p.lda, (int)p.m, (int)p.k, reinterpret_cast<float *>(w), k4, (int)p.m,
                                 p.B, p.ldb, (int)p.k, (int)p.n, reinterpret_cast<float *>(w + need_a), n4, (int)k4, s);
    if (copy_a) {
        if (!copy_b) e = tg::launch_pad_copy(p.A, p.lda, (int)p.m, (int)p.k, reinterpret_cast<float *>(w), k4, (int)p.m, s);
        p.A = reinterpret_cast<const float *>(w);
        p.lda = k4;
        w += need_a;
    }
    if (e == hipSuccess && copy_b) {
        if (!copy_a) e = tg::launch_pad_copy(p.B, p.ldb, (int)p.k, (int)p.n, reinterpret_cast<float *>(w), n4, (int)k4, s);
        p.B = reinterpret_cast<const float *>(w);
        p.ldb = n4;
        p.nb = n4;
        w += need_b;
    }
    if (e != hipSuccess) return fail(TG_ERR_HIP, std::string("copy launch failed: ") + hipGetErrorString(e));
    ws = w;
    ws_bytes -= need_a + need_b;
    p.k = k4;
    *tag = copy_a && copy_b ? "+alignAB" : (copy_a ? "+alignA" : "+alignB");
    return validate(p);   // the alignment class of the copies
}

// Time of the packing pass over a rows x cols operand (seconds): it reads whole lines along whichever axis has the
// smaller stride (64 x 64 tiles through LDS), so an element costs min(4 x that stride, 128) bytes of line traffic,
// and it writes 4 bytes.  Measured: 1024 x 1024 at element stride 32 (128 MiB of lines) 26 us.
double pack_seconds(int64_t rows, int64_t cols, int64_t rs, int64_t cs) {
    const double line = std::min<double>(4.0 * std::min(rs, cs), 128.0);
    const double elems = (double)rows * cols;
    return 2.5e-6 + std::max(elems * line / 5.5e12, elems * 8.0 / 4e12);
}

// A gathering variant asks for every element of the strided operand once per tile that uses it; the packing pass
// asks once in all and leaves a unit-stride problem.  With room for the copies the cost model says which is faster
// (1024^3 with A at element stride 32: fused 44 us, packed 50 us; 2048^3: fused 434 us, packed 230 us); the fused
// form, which leaves the workspace alone, keeps a margin that covers the model's error on both.  Caller holds g_mutex.
bool packing_is_faster(const Problem &p, const Config &fused_cfg, void *ws, size_t ws_bytes) {
    const bool want_a = p.csa != 1 && p.n > kPackMinReuse, want_b = p.csb != 1 && p.m > kPackMinReuse;
    const size_t need_a = want_a ? pack_bytes(p.m, p.k) : 0, need_b = want_b ? pack_bytes(p.k, p.n) : 0;
    if (!(want_a || want_b) || ws == nullptr || need_a + need_b > ws_bytes) return false;
    Problem q = p;
    double t = 0;
    if (want_a) {
        t += pack_seconds(p.m, p.k, p.lda, p.csa);
        q.A = static_cast<const float *>(ws); q.lda = pack_ld(p.k); q.csa = 1;
    }
    if (want_b) {
        t += pack_seconds(p.k, p.n, p.ldb, p.csb);
        q.B = reinterpret_cast<const float *>(static_cast<char *>(ws) + need_a); q.ldb = pack_ld(p.n); q.csb = 1;
    }
    Config c;
    if (validate(q) != TG_OK || choose(q, ws_bytes - need_a - need_b, &c) != TG_OK) return false;
    return t + heuristic_seconds(q, c) < 0.95 * heuristic_seconds(p, fused_cfg);
}

tg_status run(Problem &p, void *stream) {
    tg_status st = validate(p);
    if (st != TG_OK) return st;
    if (p.batch == 0 || p.m == 0 || p.n == 0) { t_last_config.clear(); t_last_pending = false; return TG_OK; }
    st = check_device();
    if (st != TG_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (p.k == 0) { t_last_config = "zero_fill"; t_last_pending = false; return zero_fill(p, s); }
    void *ws;
    size_t ws_bytes;
    {
        std::lock_guard<std::mutex> lk(g_mutex);
        ws = g_ws;
        ws_bytes = g_ws_bytes;
    }
    // Element-strided or transposed operands: when the workspace has room, gather each such
    // operand once into a packed row-major copy and multiply that with the unit-stride kernels
    // (a strided element costs a whole cache line per fetch; the tile kernels would fetch it once
    // per tile column or row).  Without room the predicated kernels gather on the fly.
    // A variant that reads the operands as they lie (transposed: 16-byte loads along the other axis; element
    // strides: 4-byte gathers straight into LDS, several K tiles ahead) needs neither the workspace nor a second
    // pass: when the choice for the problem as it stands is such a variant, nothing is packed.
    // (Not for an operand that would have to be gathered across its unit-stride axis, i.e. a transposed operand off
    // the 16-byte grid: the gather's lanes run along k of A / n of B, so there it touches a line per element where
    // the packing pass reads whole lines; such an operand is packed when there is room.)
    const char *packed = "";
    bool fused = false;
    if (!p.unit()) {
        std::lock_guard<std::mutex> lk(g_mutex);
        read_env_once();
        Config c0;
        if (g_forced) fused = config_valid(p, g_force_cfg, ws_bytes) && !tg::kernel(g_force_cfg.kernel).edge;
        else fused = choose(p, ws_bytes, &c0) == TG_OK && !tg::kernel(c0.kernel).edge &&
                     !(p.a_class() == 2 && p.lda < p.csa) && !(p.b_class() == 2 && p.ldb < p.csb);
        if (fused && !g_forced && p.batch == 1 && (tg::kernel(c0.kernel).amode == 2 || tg::kernel(c0.kernel).bmode == 2))
            fused = !packing_is_faster(p, c0, ws, ws_bytes);
    }
    if (!p.unit() && p.batch == 1 && !fused) {
        const bool want_a = p.csa != 1 && p.n > kPackMinReuse, want_b = p.csb != 1 && p.m > kPackMinReuse;
        const size_t need_a = want_a ? pack_bytes(p.m, p.k) : 0, need_b = want_b ? pack_bytes(p.k, p.n) : 0;
        if ((want_a || want_b) && need_a + need_b <= ws_bytes &&
            ceil_div(p.m, 64) * ceil_div(p.k, 64) <= INT32_MAX && ceil_div(p.k, 64) * ceil_div(p.n, 64) <= INT32_MAX) {
            char *w = static_cast<char *>(ws);
            hipError_t e = hipSuccess;
            if (want_a) {
                const int64_t ld = pack_ld(p.k);
                e = tg::launch_pack(p.A, p.lda, p.csa, reinterpret_cast<float *>(w), ld, (int)p.m, (int)p.k, s);
                p.A = reinterpret_cast<const float *>(w); p.lda = ld; p.csa = 1;
                w += need_a;
            }
            if (e == hipSuccess && want_b) {
                const int64_t ld = pack_ld(p.n);
                e = tg::launch_pack(p.B, p.ldb, p.csb, reinterpret_cast<float *>(w), ld, (int)p.k, (int)p.n, s);
                p.B = reinterpret_cast<const float *>(w); p.ldb = ld; p.csb = 1;
                w += need_b;
            }
            if (e != hipSuccess) return fail(TG_ERR_HIP, std::string("pack launch failed: ") + hipGetErrorString(e));
            ws = w;
            ws_bytes -= need_a + need_b;
            packed = want_a && want_b ? "+packAB" : (want_a ? "+packA" : "+packB");
            st = validate(p);   // recompute the alignment class of the packed problem
            if (st != TG_OK) return st;
        }
    }
    std::string copied;
    if (packed[0] == '\0') {   // (operands gathered just above are not copied a second time)
        st = align_operands(p, ws, ws_bytes, s, &copied);
        if (st != TG_OK) return st;
    }
    Config c;
    {
        std::lock_guard<std::mutex> lk(g_mutex);
        st = choose(p, ws_bytes, &c);
    }
    if (st != TG_OK) return st;
    st = launch(p, c, ws, s);
    if (st == TG_OK) {   // formatted only when tg_last_config() asks: a call must not pay for a string it may never show
        t_last_cfg = c;
        t_last_tags[0] = packed;
        t_last_tags[1] = copied.empty() ? "" : (copied == "+alignAB" ? "+alignAB" : (copied == "+alignA" ? "+alignA" : "+alignB"));
        t_last_pending = true;
    }
    return st;
}

// tg_sgemm_splitk_static: the split-K form of the product for callers that cannot allocate.  The partial
// products live in the library's fixed-size device array instead of a caller workspace; nothing here (or
// below it) allocates or frees device memory.  The configuration is the split-K candidate (two or more K
// ranges, one launch plus the reduction) that the cost model ranks first for a workspace of that size,
// memoised per shape class; a forced configuration is honoured when it is such a split.
std::map<ShapeKey, Config> g_static_choice;

bool static_split_ok(const Config &c) {
    const KernelInfo &ki = tg::kernel(c.kernel);
    return c.splits >= 2 && c.tail == 0 && ki.kind == tg::KIND_TILE && !ki.precut && !ki.pieces;
}

tg_status run_splitk_static(Problem &p, void *stream) {
    tg_status st = validate(p);
    if (st != TG_OK) return st;
    if (p.batch == 0 || p.m == 0 || p.n == 0) { t_last_config.clear(); t_last_pending = false; return TG_OK; }
    // two partial products are the least a split needs: sizes beyond that are refused before any GPU call
    if (ws_need(p, 2) > tg::kStaticScratchBytes)
        return fail(TG_ERR_WORKSPACE, "problem too large for the static scratch: 2 * m * n * 4 bytes = " +
                                          std::to_string(ws_need(p, 2)) + " exceeds " + std::to_string(tg::kStaticScratchBytes));
    st = check_device();
    if (st != TG_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (p.k == 0) { t_last_config = "zero_fill"; t_last_pending = false; return zero_fill(p, s); }
    void *ws = nullptr;
    const hipError_t e = tg::static_scratch(&ws);
    if (e != hipSuccess) return fail(TG_ERR_HIP, std::string("address of the static scratch: ") + hipGetErrorString(e));
    Config c;
    {
        std::lock_guard<std::mutex> lk(g_mutex);
        read_env_once();
        if (g_forced) {
            std::string why;
            if (!config_valid(p, g_force_cfg, tg::kStaticScratchBytes, &why))
                return fail(ws_total(p, g_force_cfg) > tg::kStaticScratchBytes ? TG_ERR_WORKSPACE : TG_ERR_INVALID_ARG,
                            "forced configuration " + spec_of(g_force_cfg) + " is not valid here: " + why);
            if (!static_split_ok(g_force_cfg))
                return fail(TG_ERR_INVALID_ARG, "forced configuration " + spec_of(g_force_cfg) + " is not a plain split-K of an fp32 tile kernel");
            c = g_force_cfg;
        } else {
            auto hit = g_static_choice.find(key_of(p));
            if (hit != g_static_choice.end() && config_valid(p, hit->second, tg::kStaticScratchBytes)) {
                c = hit->second;
            } else {
                bool found = false;
                for (const Config &cand : candidates(p, tg::kStaticScratchBytes))   // cheapest by the cost model first
                    if (static_split_ok(cand)) { c = cand; found = true; break; }
                if (!found)
                    return fail(TG_ERR_UNSUPPORTED, "no split-K configuration fits this problem (K shorter than two K tiles per "
                                                    "range, or the tile grid already fills the chip): use tg_sgemm");
                if (g_static_choice.size() >= 4096) g_static_choice.clear();
                g_static_choice[key_of(p)] = c;
            }
        }
    }
    st = launch(p, c, ws, s);
    if (st == TG_OK) {
        t_last_cfg = c;
        t_last_tags[0] = t_last_tags[1] = "";
        t_last_pending = true;
    }
    return st;
}

// Is the problem launch-bound, i.e. would back-to-back calls only measure the host's launch rate?  Decided from the
// cost model's device time of the candidate it ranks first (its estimate less the launch cost it includes), never
// from a measured per-call time: under a profiler or on a busy host every call takes tens of microseconds, and a
// classification made from that would skip the device-time measurement exactly when it is needed.
constexpr double kLaunchBoundDeviceSeconds = 12e-6;
bool launch_bound_problem(const Problem &p, const std::vector<Config> &cands) {
    return !cands.empty() && heuristic_seconds(p, cands.front()) - 4e-6 < kLaunchBoundDeviceSeconds;
}

// The timing tuner behind tg_tune: one object per call.
//   1. sweep: every candidate (sorted by the cost model) is timed briefly; one whose lower bound
//      already exceeds the best time seen is skipped (the branch-and-bound cut of Sec. 5.1 of
//      the paper, applied to a flat candidate set);
//   2. refine: tile-order group, cap on workgroups per CU and (persistent variants) workgroups
//      per CU of the winner;
//   3. final round among the leading kernel variants, with timings that can tell them apart.
// Every candidate's result is compared with the first candidate's before it may lead (result check below).
class Tuner {
  public:
    Tuner(const Problem &p, void *ws, size_t ws_bytes, hipStream_t stream, int reps)
        : p_(p), ws_(ws), ws_bytes_(ws_bytes), s_(stream), reps_(reps), log_(getenv("TG_LOG") != nullptr) {
        events_ok_ = hipEventCreate(&ev0_) == hipSuccess && hipEventCreate(&ev1_) == hipSuccess;
        // test switches (documented in tgemm.h): a host-side delay after every timed launch, in microseconds, and a
        // deliberately spoilt reference for the result check
        if (const char *d = getenv("TG_TUNE_TEST_HOST_DELAY_US")) host_delay_us_ = atof(d);
        spoil_reference_ = getenv("TG_TUNE_TEST_SPOIL_REFERENCE") != nullptr;
    }
    ~Tuner() {
        if (ev0_) (void)hipEventDestroy(ev0_);
        if (ev1_) (void)hipEventDestroy(ev1_);
    }
    Tuner(const Tuner &) = delete;
    Tuner &operator=(const Tuner &) = delete;

    tg_status run(Config *best, double *best_us) {
        if (!events_ok_) return fail(TG_ERR_HIP, "hipEventCreate failed");
        const std::vector<Config> cands = candidates(p_, ws_bytes_);
        if (cands.empty()) return fail(TG_ERR_INTERNAL, "no kernel variant is valid for this problem");
        launch_bound_ = launch_bound_problem(p_, cands);
        prepare_check();
        warm_up(cands);
        sweep(cands);
        if (best_.kernel < 0) return fail(TG_ERR_HIP, "every candidate failed to run: " + last_err_);
        if (tg::kernel(best_.kernel).kind == tg::KIND_TILE) {
            refine_group();
            refine_occupancy();
            refine_persistence();
        }
        final_round();
        // A candidate whose product differs from the first candidate's is a defect of the library, not a tuning result:
        // nothing is cached and the call says which configurations disagree.
        if (!disagree_.empty())
            return fail(TG_ERR_INTERNAL, "result check: " + disagree_ + " (reference: " + spec_of(ref_cfg_) + "); nothing cached");
        *best = best_;
        *best_us = best_us_;
        return TG_OK;
    }

  private:
    // ---- result check -------------------------------------------------------------------------------------------
    // The first candidate that runs leaves its product in C; every step-th row of it is copied into the library's
    // static scratch (step such that the copy fits; 1 for products up to about 8 M elements).  Every later candidate's
    // product is compared with it on those rows: two results that each meet the benchmark's bar (relative Frobenius
    // error <= 1e-6 against the exact product, Sec. 5.2 definition) differ by at most 2e-6 in that norm; the check
    // allows 4e-6 and no non-finite value.  A candidate that fails is dropped and reported.
    void prepare_check() {
        void *base = nullptr;
        if (tg::static_scratch(&base) != hipSuccess || base == nullptr) return;   // no check without the scratch
        const size_t room = tg::kStaticScratchBytes - kPartialBytes;
        const double need = 4.0 * (double)p_.batch * (double)p_.m * (double)p_.n;
        step_ = (int)std::min<double>(std::max(1.0, std::ceil(need / (double)room)), (double)p_.m);
        const int64_t rows = ceil_div(p_.m, step_);
        if ((double)p_.batch * rows * p_.n * 4.0 > (double)room) return;          // (a single row too long: no check)
        ref_ = static_cast<float *>(base);
        partial_ = reinterpret_cast<double *>(static_cast<char *>(base) + room);
    }

    void take_reference(const Config &c) {
        if (!ref_ || have_ref_) return;
        if (launch(p_, c, ws_, s_) != TG_OK) return;
        hipError_t e = tg::launch_snapshot_rows(p_.C, p_.ldc, p_.strideC, (int)p_.batch, (int)p_.m, (int)p_.n, step_, ref_, s_);
        if (e == hipSuccess && spoil_reference_) {
            static const float kBogus = 1.0e30f;
            e = hipMemcpyAsync(ref_, &kBogus, sizeof kBogus, hipMemcpyHostToDevice, s_);
        }
        if (e == hipSuccess) e = hipStreamSynchronize(s_);
        if (e != hipSuccess) { (void)hipGetLastError(); return; }
        have_ref_ = true;
        ref_cfg_ = c;
    }

    // true: agrees with the reference (or no check is possible)
    bool agrees(const Config &c) {
        if (!have_ref_) return true;
        // C still holds an earlier candidate's (correct) product: filled with NaN first, so that a candidate which
        // leaves part of C unwritten cannot pass on what was there
        for (int64_t b = 0; b < p_.batch; ++b)
            if (hipMemset2DAsync(p_.C + b * p_.strideC, (size_t)p_.ldc * sizeof(float), 0xFF, (size_t)p_.n * sizeof(float), (size_t)p_.m, s_) != hipSuccess) {
                (void)hipGetLastError();
                return true;
            }
        if (launch(p_, c, ws_, s_) != TG_OK) return true;   // (a launch failure is reported by the timing path)
        double host[3 * tg::kCheckBlocks];
        hipError_t e = tg::launch_compare_rows(p_.C, p_.ldc, p_.strideC, (int)p_.batch, (int)p_.m, (int)p_.n, step_, ref_, partial_, s_);
        if (e == hipSuccess) e = hipMemcpyAsync(host, partial_, sizeof host, hipMemcpyDeviceToHost, s_);
        if (e == hipSuccess) e = hipStreamSynchronize(s_);
        if (e != hipSuccess) { (void)hipGetLastError(); return true; }
        double d2 = 0, r2 = 0, bad = 0;
        for (int b = 0; b < tg::kCheckBlocks; ++b) { d2 += host[3 * b]; r2 += host[3 * b + 1]; bad += host[3 * b + 2]; }
        const bool ok = bad == 0 && d2 <= (4e-6 * 4e-6) * r2;
        if (!ok) {
            char buf[256];
            snprintf(buf, sizeof buf, "%s%s differs (relative Frobenius difference %.3g, %.0f non-finite)", disagree_.empty() ? "" : "; ",
                     spec_of(c).c_str(), r2 > 0 ? std::sqrt(d2 / r2) : 0.0, bad);
            disagree_ += buf;
            if (log_) fprintf(stderr, "tgemm tune: %s\n", buf);
        }
        return ok;
    }

    void host_delay() const {
        if (host_delay_us_ <= 0) return;
        const auto until = std::chrono::steady_clock::now() + std::chrono::duration<double, std::micro>(host_delay_us_);
        while (std::chrono::steady_clock::now() < until) {}
    }

    // An idle GPU takes its time to reach its clock under load (measured on MI355X: the first configuration timed in a
    // fresh process read 43 us after 50 ms of launches, 37 us later on), and the sweep times the model's favourites
    // first: they would be the ones to lose.  The first candidate that runs is launched for 0.2 s before anything is timed.
    void warm_up(const std::vector<Config> &cands) {
        const auto until = std::chrono::steady_clock::now() + std::chrono::milliseconds(200);
        for (const Config &c : cands) {
            if (launch(p_, c, ws_, s_) != TG_OK) { (void)hipGetLastError(); continue; }
            while (std::chrono::steady_clock::now() < until) {
                for (int i = 0; i < 16; ++i)
                    if (launch(p_, c, ws_, s_) != TG_OK) { (void)hipGetLastError(); break; }
                if (hipStreamSynchronize(s_) != hipSuccess) { (void)hipGetLastError(); break; }
            }
            break;
        }
        (void)hipStreamSynchronize(s_);
    }

    // One brief timing: warm-up launch, then `n` back-to-back launches between two events.
    // Short kernels are repeated more often (until about 0.3 ms is covered) so that launch
    // jitter does not decide between candidates.
    tg_status time_briefly(const Config &c, double *usec) {
        tg_status r = launch(p_, c, ws_, s_);   // warm-up (also loads the code object)
        if (r != TG_OK) return r;
        int n = reps_;
        double best_of = 1e300;
        for (int round = 0; round < 3; ++round) {
            hipError_t e = hipEventRecord(ev0_, s_);
            for (int i = 0; i < n && r == TG_OK; ++i) { r = launch(p_, c, ws_, s_); host_delay(); }
            if (e == hipSuccess) e = hipEventRecord(ev1_, s_);
            if (e == hipSuccess) e = hipEventSynchronize(ev1_);
            if (r != TG_OK) return r;
            float ms = 0.f;
            if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev0_, ev1_);
            if (e != hipSuccess) return fail(TG_ERR_HIP, std::string("tuning run failed: ") + hipGetErrorString(e));
            const double us = 1e3 * ms / n;
            best_of = std::min(best_of, us);
            if (round >= 1 && (us * n >= 300.0 || n >= 64)) break;   // at least two rounds, long enough
            n = std::min<int>(64, std::max<int>(n * 2, (int)(300.0 / std::max(us, 1.0)) + 1));
        }
        *usec = best_of;
        return TG_OK;
    }

    // Times `c`, records it and makes it the leader when it beats the best by `margin`.  `check`: a kernel variant not
    // seen before, whose product is compared with the reference first (the refinements re-run a variant that passed).
    void consider(const Config &c, double margin, bool check = false) {
        // (the refinements vary one parameter of a valid configuration; not every value stays valid: the walking
        // row-panel variants need the tiles to divide over the workgroups)
        if (!config_valid(p_, c, ws_bytes_)) return;
        double us = 0;
        if (time_briefly(c, &us) != TG_OK) {
            last_err_ = t_error;
            (void)hipGetLastError();   // clear the error so the next candidate starts clean
            return;
        }
        if (check) {
            if (!have_ref_) take_reference(c);
            else if (!agrees(c)) return;
        }
        if (log_) fprintf(stderr, "tgemm tune: %-44s %.2f us\n", spec_of(c).c_str(), us);
        seen_.emplace_back(us, c);
        if (us < best_us_ * margin) { best_us_ = us; best_ = c; }
    }

    void sweep(const std::vector<Config> &cands) {
        for (const Config &c : cands) {
            const double lb_us = 1e6 * lower_bound_seconds(p_, c);
            if (lb_us >= best_us_) {
                if (log_) fprintf(stderr, "tgemm tune: %-44s pruned (bound %.1f us >= best %.1f us)\n", spec_of(c).c_str(), lb_us, best_us_);
                continue;
            }
            consider(c, 1.0, true);
        }
    }

    void refine_group() {
        static const int kGroups[] = {1, 2, 4, 16, 32};
        const int tiles_m = (int)ceil_div(p_.m, tg::kernel(best_.kernel).BM);
        const Config base = best_;
        for (int g : kGroups) {
            if (g >= 2 * tiles_m && g != 1) continue;
            Config c = base;
            c.group = g;
            consider(c, 0.995);   // (another order must win by more than the timing noise: it also changes the L2 traffic)
        }
    }

    void refine_occupancy() {
        const Config base = best_;
        for (int occ = 1; occ <= 4; ++occ) {
            Config c = base;
            c.occ = occ;
            consider(c, 0.995);
        }
    }

    void refine_persistence() {
        const Config base = best_;
        for (int per_cu = 1; per_cu <= 4 && tg::kernel(base.kernel).persistent; ++per_cu) {
            Config c = base;
            c.persist = per_cu;
            consider(c, 0.995, true);   // (checked again: the number of workgroups decides which of them takes which tile)
        }
    }

    // `n` back-to-back launches on the caller's stream; microseconds per launch, or < 0 on failure.
    double time_run(const Config &c, int n) {
        tg_status r = TG_OK;
        hipError_t e = hipEventRecord(ev0_, s_);
        for (int j = 0; j < n && r == TG_OK; ++j) { r = launch(p_, c, ws_, s_); host_delay(); }
        if (e == hipSuccess) e = hipEventRecord(ev1_, s_);
        if (e == hipSuccess) e = hipEventSynchronize(ev1_);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev0_, ev1_);
        if (e != hipSuccess || r != TG_OK) {
            (void)hipGetLastError();
            return -1.0;
        }
        return 1e3 * ms / n;
    }

    // Device time per launch: 32 launches captured into a graph on `ts`, replayed four times.
    double time_graph(const Config &c, hipStream_t ts) {
        const int per_graph = 32, replays = 4;
        hipGraph_t graph = nullptr;
        hipGraphExec_t exec = nullptr;
        tg_status r = TG_OK;
        bool ok = hipStreamBeginCapture(ts, hipStreamCaptureModeThreadLocal) == hipSuccess;
        for (int j = 0; ok && j < per_graph && r == TG_OK; ++j) r = launch(p_, c, ws_, ts);
        ok = ok && hipStreamEndCapture(ts, &graph) == hipSuccess && r == TG_OK && graph != nullptr;
        ok = ok && hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0) == hipSuccess;
        ok = ok && hipGraphLaunch(exec, ts) == hipSuccess;   // warm-up replay
        float ms = 0.f;
        if (ok) {
            ok = hipEventRecord(ev0_, ts) == hipSuccess;
            for (int j = 0; j < replays && ok; ++j) ok = hipGraphLaunch(exec, ts) == hipSuccess;
            ok = ok && hipEventRecord(ev1_, ts) == hipSuccess;
            ok = hipEventSynchronize(ev1_) == hipSuccess && ok;
            ok = ok && hipEventElapsedTime(&ms, ev0_, ev1_) == hipSuccess;
        }
        if (exec) (void)hipGraphExecDestroy(exec);
        if (graph) (void)hipGraphDestroy(graph);
        if (!ok) {
            (void)hipGetLastError();
            (void)hipStreamSynchronize(ts);
            return -1.0;
        }
        return 1e3 * ms / (per_graph * replays);
    }

    // Long kernels: the leaders are often within the noise of the brief timings (1 % at 4096^3),
    // so the three fastest kernel variants within 2 % of the best are timed again, alternating,
    // with longer runs (>= 10 launches and >= 2 ms each).
    // Launch-bound problems (modelled device time under 12 us, see launch_bound_problem): back-to-back calls
    // only measure the host's launch rate, which is the same for every candidate, so up to six variants within
    // 25 % (every variant seen, when the host is so slow that all per-call times are alike) are timed as replays
    // of a captured graph on a private stream, i.e. by their device time.  The best of two such runs decides.
    void final_round() {
        const bool launch_bound = launch_bound_;
        const size_t max_finalists = launch_bound ? 4 : 3;
        const double window = launch_bound ? 1.25 : 1.02;
        std::stable_sort(seen_.begin(), seen_.end(),
                         [](const std::pair<double, Config> &a, const std::pair<double, Config> &b) { return a.first < b.first; });
        std::vector<Config> finalists{best_};
        auto add = [&](const Config &c) {      // one entry per kernel variant: its fastest setting so far
            for (const Config &f : finalists)
                if (f.kernel == c.kernel) return;
            finalists.push_back(c);
        };
        for (const auto &sc : seen_) {
            if (finalists.size() >= max_finalists || sc.first > best_us_ * window) break;
            add(sc.second);
        }
        if (launch_bound) {
            // the per-call times of a launch-bound problem say little (nothing at all on a slow host): the four
            // variants the cost model ranks first are timed by their device time as well
            std::vector<std::pair<double, Config>> by_model;
            for (const auto &sc : seen_) by_model.emplace_back(heuristic_seconds(p_, sc.second), sc.second);
            std::stable_sort(by_model.begin(), by_model.end(),
                             [](const std::pair<double, Config> &a, const std::pair<double, Config> &b) { return a.first < b.first; });
            for (size_t i = 0, taken = 0; i < by_model.size() && taken < 4; ++i) {
                const size_t before = finalists.size();
                add(by_model[i].second);
                taken += finalists.size() > before || by_model[i].second.kernel == best_.kernel ? 1 : 0;
            }
        }
        if (finalists.size() < 2) return;

        hipStream_t ts = nullptr;   // private stream: the caller's may be the null stream, which cannot be captured
        const bool use_graph = launch_bound && hipStreamSynchronize(s_) == hipSuccess && hipStreamCreate(&ts) == hipSuccess;
        const int n = std::min<int>(256, std::max<int>(10, (int)(2000.0 / std::max(best_us_, 1.0)) + 1));
        std::vector<double> fin(finalists.size(), 1e300);
        for (int pass = 0; pass < 2; ++pass)
            for (size_t i = 0; i < finalists.size(); ++i) {
                const double us = use_graph ? time_graph(finalists[i], ts) : time_run(finalists[i], n);
                if (us >= 0) fin[i] = std::min(fin[i], us);
            }
        if (ts) {
            (void)hipStreamSynchronize(ts);
            (void)hipStreamDestroy(ts);
        }
        size_t w = 0;
        for (size_t i = 1; i < finalists.size(); ++i)
            if (fin[i] < fin[w]) w = i;
        if (fin[w] < 1e300) {
            best_ = finalists[w];
            if (!use_graph) best_us_ = fin[w];   // (a graph time is not comparable with the per-call times in the cache)
        }
        if (log_)
            for (size_t i = 0; i < finalists.size(); ++i)
                fprintf(stderr, "tgemm tune: final%s %-38s %.2f us%s\n", use_graph ? " (graph replay)" : "",
                        spec_of(finalists[i]).c_str(), fin[i], i == w ? "  <- chosen" : "");
    }

    const Problem &p_;
    void *ws_;
    size_t ws_bytes_;
    hipStream_t s_;
    int reps_;
    bool log_;
    bool events_ok_ = false;
    hipEvent_t ev0_ = nullptr, ev1_ = nullptr;
    Config best_;
    double best_us_ = 1e300;
    std::string last_err_;
    std::vector<std::pair<double, Config>> seen_;   // every configuration measured, for the final round
    bool launch_bound_ = false;
    // result check
    static constexpr size_t kPartialBytes = 16384;  // tail of the static scratch: 3 doubles per checking workgroup
    float *ref_ = nullptr;
    double *partial_ = nullptr;
    int step_ = 1;
    bool have_ref_ = false;
    Config ref_cfg_;
    std::string disagree_;
    // test switches
    double host_delay_us_ = 0;
    bool spoil_reference_ = false;
};

// The packed, aligned problem of these sizes (no operands: for queries only).
tg_status query_problem(int64_t batch, int64_t m, int64_t n, int64_t k, Problem *out) {
    if (batch <= 0 || m <= 0 || n <= 0 || k <= 0) return fail(TG_ERR_INVALID_ARG, "sizes must be positive");
    if (m > INT32_MAX || n > INT32_MAX || k > INT32_MAX || batch > INT32_MAX) return fail(TG_ERR_UNSUPPORTED, "a dimension exceeds 2^31-1");
    *out = Problem{batch, m, n, k, nullptr, k, m * k, nullptr, n, k * n, nullptr, n, m * n, false};
    out->aligned = k % 4 == 0 && n % 4 == 0;
    return TG_OK;
}

}  // namespace

extern "C" {

tg_status tg_sgemm(int64_t m, int64_t n, int64_t k, const float *A, int64_t lda, const float *B, int64_t ldb,
                   float *C, int64_t ldc, void *stream) {
    Problem p{1, m, n, k, A, lda, 0, B, ldb, 0, C, ldc, 0, false};
    return run(p, stream);
}

tg_status tg_sgemm_batched(int64_t batch, int64_t m, int64_t n, int64_t k, const float *A, int64_t lda,
                           int64_t strideA, const float *B, int64_t ldb, int64_t strideB, float *C, int64_t ldc,
                           int64_t strideC, void *stream) {
    Problem p{batch, m, n, k, A, lda, strideA, B, ldb, strideB, C, ldc, strideC, false};
    return run(p, stream);
}

tg_status tg_sgemm_strided(int64_t m, int64_t n, int64_t k, const float *A, int64_t rsa, int64_t csa, const float *B,
                           int64_t rsb, int64_t csb, float *C, int64_t ldc, void *stream) {
    Problem p{1, m, n, k, A, rsa, 0, B, rsb, 0, C, ldc, 0, false};
    p.csa = csa;
    p.csb = csb;
    return run(p, stream);
}

tg_status tg_sgemm_splitk_static(int64_t m, int64_t n, int64_t k, const float *A, int64_t lda, const float *B, int64_t ldb,
                                 float *C, int64_t ldc, void *stream) {
    Problem p{1, m, n, k, A, lda, 0, B, ldb, 0, C, ldc, 0, false};
    return run_splitk_static(p, stream);
}

tg_status tg_saxpy(int64_t n, float alpha, const float *x, const float *y, float *z, void *stream) {
    if (n < 0) return fail(TG_ERR_INVALID_ARG, "negative size");
    if (n == 0) return TG_OK;
    if (!x || !y || !z) return fail(TG_ERR_INVALID_ARG, "x, y or z is null");
    if (n > INT64_MAX / 4) return fail(TG_ERR_INVALID_ARG, "vector extent overflows int64");
    tg_status st = check_device();
    if (st != TG_OK) return st;
    hipError_t e = tg::launch_saxpy(n, alpha, x, y, z, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(TG_ERR_HIP, std::string("saxpy launch failed: ") + hipGetErrorString(e));
    return TG_OK;
}

tg_status tg_tune(int64_t batch, int64_t m, int64_t n, int64_t k, const float *A, int64_t lda, int64_t strideA,
                  const float *B, int64_t ldb, int64_t strideB, float *C, int64_t ldc, int64_t strideC,
                  void *stream, int reps) {
    Problem p{batch, m, n, k, A, lda, strideA, B, ldb, strideB, C, ldc, strideC, false};
    tg_status st = validate(p);
    if (st != TG_OK) return st;
    if (p.batch == 0 || p.m == 0 || p.n == 0 || p.k == 0) return run(p, stream);
    st = check_device();
    if (st != TG_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);

    void *ws;
    size_t ws_bytes;
    {
        std::lock_guard<std::mutex> lk(g_mutex);
        ws = g_ws;
        ws_bytes = g_ws_bytes;
    }
    std::string copied;
    st = align_operands(p, ws, ws_bytes, s, &copied);   // as a call would: the tuned entry is for the copies' shape class
    if (st != TG_OK) return st;
    Config best;
    double best_us = 0;
    {
        Tuner tuner(p, ws, ws_bytes, s, reps <= 0 ? 5 : reps);
        st = tuner.run(&best, &best_us);
    }
    if (st != TG_OK) return st;

    st = launch(p, best, ws, s);   // leave C holding the product computed by the winner
    hipError_t e = hipStreamSynchronize(s);
    if (st != TG_OK) return st;
    if (e != hipSuccess) return fail(TG_ERR_HIP, std::string("hipStreamSynchronize: ") + hipGetErrorString(e));
    {
        std::lock_guard<std::mutex> lk(g_mutex);
        read_env_once();
        g_cache[key_of(p)] = TunedEntry{best, best_us};
        const char *path = getenv("TG_TUNE_CACHE");
        if (path && *path && save_cache_locked(path) != TG_OK)
            fprintf(stderr, "tgemm: could not write TG_TUNE_CACHE: %s\n", t_error.c_str());
    }
    t_last_config = spec_of(best) + copied;
    t_last_pending = false;
    return TG_OK;
}

tg_status tg_set_workspace(void *dev_ptr, size_t bytes) {
    if ((dev_ptr == nullptr) != (bytes == 0)) return fail(TG_ERR_INVALID_ARG, "workspace pointer and size must both be set or both be empty");
    if (reinterpret_cast<uintptr_t>(dev_ptr) & 15u) return fail(TG_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
    std::lock_guard<std::mutex> lk(g_mutex);
    g_ws = dev_ptr;
    g_ws_bytes = bytes;
    return TG_OK;
}

size_t tg_workspace_bytes(int64_t batch, int64_t m, int64_t n, int64_t k) {
    if (batch <= 0 || m <= 0 || n <= 0 || k <= 0) return 0;
    if (m > INT32_MAX || n > INT32_MAX || k > INT32_MAX || batch > INT32_MAX) return 0;
    Problem p{batch, m, n, k, nullptr, k, m * k, nullptr, n, k * n, nullptr, n, m * n, true};
    size_t need = 0;
    for (const Config &c : candidates(p, SIZE_MAX)) need = std::max(need, ws_total(p, c));
    return need;
}

size_t tg_strided_workspace_bytes(int64_t m, int64_t n, int64_t k, int64_t csa, int64_t csb) {
    if (m <= 0 || n <= 0 || k <= 0 || csa < 1 || csb < 1) return 0;
    if (m > INT32_MAX || n > INT32_MAX || k > INT32_MAX) return 0;
    size_t need = tg_workspace_bytes(1, m, n, k);
    if (csa != 1) need += pack_bytes(m, k);
    if (csb != 1) need += pack_bytes(k, n);
    return need;
}

tg_status tg_set_math(int mode) {
    if (mode != TG_MATH_FP32_MFMA && mode != TG_MATH_BF16_PIECES) return fail(TG_ERR_INVALID_ARG, "unknown math mode");
    std::lock_guard<std::mutex> lk(g_mutex);
    if (mode != g_math) g_heuristic_choice.clear();
    g_math = mode;
    return TG_OK;
}

int tg_get_math(void) {
    std::lock_guard<std::mutex> lk(g_mutex);
    return g_math;
}

tg_status tg_force_config(const char *spec) {
    std::lock_guard<std::mutex> lk(g_mutex);
    g_env_read = true;   // an explicit call overrides the environment
    if (!spec || !*spec) { g_forced = false; return TG_OK; }
    Config c;
    std::string why;
    if (!parse_spec(spec, c, why)) return fail(TG_ERR_INVALID_ARG, "bad configuration spec: " + why);
    g_forced = true;
    g_force_cfg = c;
    return TG_OK;
}

tg_status tg_get_config(int64_t batch, int64_t m, int64_t n, int64_t k, char *buf, size_t len) {
    if (!buf || len == 0) return fail(TG_ERR_INVALID_ARG, "no output buffer");
    Problem p;
    tg_status st = query_problem(batch, m, n, k, &p);
    if (st != TG_OK) return st;
    Config c;
    {
        std::lock_guard<std::mutex> lk(g_mutex);
        st = choose(p, g_ws_bytes, &c);
    }
    if (st != TG_OK) return st;
    const std::string s = spec_of(c);
    if (s.size() + 1 > len) return fail(TG_ERR_INVALID_ARG, "output buffer too small");
    memcpy(buf, s.c_str(), s.size() + 1);
    return TG_OK;
}

const char *tg_last_config(void) {
    if (t_last_pending) {
        t_last_config = spec_of(t_last_cfg) + t_last_tags[0] + t_last_tags[1];
        t_last_pending = false;
    }
    return t_last_config.c_str();
}

int tg_num_candidates(int64_t batch, int64_t m, int64_t n, int64_t k) {
    Problem p;
    if (query_problem(batch, m, n, k, &p) != TG_OK) return -1;
    std::lock_guard<std::mutex> lk(g_mutex);
    return (int)candidates(p, g_ws_bytes).size();
}

tg_status tg_candidate(int64_t batch, int64_t m, int64_t n, int64_t k, int idx, char *spec, size_t len,
                       double *lower_bound_us, double *model_us) {
    if (!spec || len == 0) return fail(TG_ERR_INVALID_ARG, "no output buffer");
    Problem p;
    tg_status st = query_problem(batch, m, n, k, &p);
    if (st != TG_OK) return st;
    std::vector<Config> cands;
    {
        std::lock_guard<std::mutex> lk(g_mutex);
        cands = candidates(p, g_ws_bytes);
    }
    if (idx < 0 || idx >= (int)cands.size()) return fail(TG_ERR_INVALID_ARG, "candidate index out of range");
    const std::string s = spec_of(cands[idx]);
    if (s.size() + 1 > len) return fail(TG_ERR_INVALID_ARG, "output buffer too small");
    memcpy(spec, s.c_str(), s.size() + 1);
    if (lower_bound_us) *lower_bound_us = 1e6 * lower_bound_seconds(p, cands[idx]);
    if (model_us) *model_us = 1e6 * heuristic_seconds(p, cands[idx]);
    return TG_OK;
}

int tg_tune_is_launch_bound(int64_t batch, int64_t m, int64_t n, int64_t k) {
    Problem p;
    if (query_problem(batch, m, n, k, &p) != TG_OK) return -1;
    std::lock_guard<std::mutex> lk(g_mutex);
    return launch_bound_problem(p, candidates(p, g_ws_bytes)) ? 1 : 0;
}

int tg_num_kernels(void) { return tg::num_kernels(); }

tg_status tg_kernel_name(int idx, char *buf, size_t len) {
    if (idx < 0 || idx >= tg::num_kernels() || !buf) return fail(TG_ERR_INVALID_ARG, "kernel index out of range");
    const char *n = tg::kernel(idx).name;
    if (strlen(n) + 1 > len) return fail(TG_ERR_INVALID_ARG, "output buffer too small");
    memcpy(buf, n, strlen(n) + 1);
    return TG_OK;
}

tg_status tg_save_tune_cache(const char *path) {
    if (!path) return fail(TG_ERR_INVALID_ARG, "path is null");
    std::lock_guard<std::mutex> lk(g_mutex);
    return save_cache_locked(path);
}

tg_status tg_load_tune_cache(const char *path) {
    if (!path) return fail(TG_ERR_INVALID_ARG, "path is null");
    std::lock_guard<std::mutex> lk(g_mutex);
    return load_cache_locked(path);
}

void tg_clear_tune_cache(void) {
    std::lock_guard<std::mutex> lk(g_mutex);
    g_cache.clear();
}

const char *tg_status_string(tg_status s) {
    switch (s) {
        case TG_OK: return "TG_OK";
        case TG_ERR_INVALID_ARG: return "TG_ERR_INVALID_ARG";
        case TG_ERR_UNSUPPORTED: return "TG_ERR_UNSUPPORTED";
        case TG_ERR_WORKSPACE: return "TG_ERR_WORKSPACE";
        case TG_ERR_HIP: return "TG_ERR_HIP";
        case TG_ERR_INTERNAL: return "TG_ERR_INTERNAL";
    }
    return "TG_ERR_UNKNOWN";
}

const char *tg_last_error(void) { return t_error.c_str(); }

// (the debug flavour, whose kernels overwrite every LDS stage they give up with NaN, reports 1000000 more)
#ifdef TG_POISON_LDS
int tg_version(void) { return kVersion + 1000000; }
#else
int tg_version(void) { return kVersion; }
#endif

}  // extern "C"
