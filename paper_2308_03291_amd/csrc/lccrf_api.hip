// C ABI of the library (declared in include/lccrf.h): argument checks, workspace carving,
// choice of schedule, launches.  No allocation, no synchronisation, no host copies.
#include "../../include/lccrf.h"
#include "../../include/lccrf_instrument.h"
#include "lccrf_launch.h"

#include <atomic>
#include <mutex>

// Built-in scratch of lccrf_marginals_static: device memory inside the library's code object, one
// copy on every GPU the library is loaded on, held until the process ends.  In host code the name
// only stands for the symbol; its device address comes from hipGetSymbolAddress (static_scratch()).
#define LCCRF_STATIC_SCRATCH_BYTES (64u << 20)
static __device__ __align__(256) unsigned char scratch[LCCRF_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;

// Compute units of the current device (the device the caller's stream belongs to), asked once per device.
std::atomic<int> g_device_cus[kMaxDevices];
int current_device_cus() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
    int n = g_device_cus[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) n = 0;
        g_device_cus[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

// Device address of `scratch` on the current device, looked up once per device.
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};
void* static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

constexpr size_t kAlign = 256;
inline size_t round_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// The two process-wide tuning knobs (atomics: a reader sees the old or the new value, never a torn one).
// Polls a workgroup of the paired second pass waits for its partner (lccrf_set_pair_poll_limit).  A poll
// is one round trip to the L2 cache, a few hundred nanoseconds: the default bounds a wait to some tens
// of milliseconds, four orders of magnitude above an exchange between resident partners (under 1 us).
constexpr int kDefaultPairPollLimit = 1 << 15;
std::atomic<int> g_pair_poll_limit{kDefaultPairPollLimit};
// Polls the chain wave of the lane kernels spends on a matrix its producers have not delivered yet
// (lccrf_set_lane_poll_limit) before it continues alone in the log domain.  A poll is one LDS read.
constexpr int kDefaultLanePollLimit = 1 << 16;
std::atomic<int> g_lane_poll_limit{kDefaultLanePollLimit};
// Positions per chunk of the scan (lccrf_set_scan_chunk).  0: chosen by shape, the smallest of 8, 16 and 32 that keeps the
// chunks of the batch (one wave each in the scan's first phase) within what the chip holds at once
// (measured: short chunks win, 8 by 2.8 times on the marginals of B=1, N=128, T=32 against the
// sequential schedule, until the chunks outnumber the SIMDs, resp. twice their number at 16 tags).
std::atomic<int> g_scan_chunk_user{0};
// An entry point reads the knob once (KnobSnapshot at its top) and every use inside the call, from sizing
// the workspace to the last launch, sees that one value, whatever another thread sets meanwhile.
thread_local int t_snapshot_depth = 0;
thread_local int t_scan_chunk_user = 0;
struct KnobSnapshot {
    KnobSnapshot() {
        if (t_snapshot_depth++ == 0) t_scan_chunk_user = g_scan_chunk_user.load(std::memory_order_relaxed);
    }
    ~KnobSnapshot() { --t_snapshot_depth; }
    KnobSnapshot(const KnobSnapshot&) = delete;
    KnobSnapshot& operator=(const KnobSnapshot&) = delete;
};
inline int scan_chunk(long long B, long long N, long long T) {
    if (const int user = t_snapshot_depth > 0 ? t_scan_chunk_user : g_scan_chunk_user.load(std::memory_order_relaxed))
        return user;
    // 33 .. 64 tags: a chunk's product takes a workgroup of three or four waves that fills a compute unit, so
    // the chunks should not outnumber the compute units (measured: B=1, N=128, T=48 is best at 8, B=32, N=256
    // and B=8, N=1024 at 32)
    const long long cap = T > 32 ? 256 : T > 16 ? 1024 : 2048;
    for (int c = 8; c < 32; c *= 2)
        if (B * ((N + c - 1) / c) <= cap) return c;
    return 32;
}

// The chunk of the max-plus scan: the sum scan's up to 16 tags; at 17 .. 32 tags its chunk products hold two waves a
// SIMD (one workgroup each), which hide what a lone wave waits for: up to 2048 chunks (B=8 N=4096 T=32: chunk
// products 210 us with 1024 chunks of 32, 130 us with 2048 of 16; a third wave a SIMD, which needs single LDS tiles
// and a shallower ring of loads, cost more than it hid: 160 us).
inline int scan_chunk_max(long long B, long long N, long long T) {
    if (T <= 16) return scan_chunk(B, N, T);
    if (const int user = t_snapshot_depth > 0 ? t_scan_chunk_user : g_scan_chunk_user.load(std::memory_order_relaxed))
        return user;
    for (int c = 8; c < 32; c *= 2)
        if (B * ((N + c - 1) / c) <= 2048) return c;
    return 32;
}

struct SumWorkspace {
    size_t ua, ub, Oa, Ob, mail, failed;
    size_t Pl, rel, base, Fv, OF, Gv, OG;  // chunked scan (T <= 32 only, else empty)
    size_t Pl2, rel2, base2, Fv2, OF2, Gv2, OG2;  // its group level (many chunks only, else empty)
    size_t lz64, ha, hb, hoff;             // log-probability, entropy and cross-entropy queries
    size_t ent, lzf;                       // entropy under the scan: per-chunk sums, logZ as float
    size_t maps, winmaps;                  // sampling: the map of every position, [B][N][T] bytes; of every window
    size_t total;
};
inline SumWorkspace sum_workspace(size_t B, size_t N, size_t T) {
    SumWorkspace w;
    size_t off = 0;
    const size_t chunk = (size_t)scan_chunk((long long)B, (long long)N, (long long)T);
    w.ua = off; off += round_up(B * N * T * sizeof(float));
    w.ub = off; off += round_up(B * N * T * sizeof(float));
    w.Oa = off; off += round_up(B * N * sizeof(double));
    w.Ob = off; off += round_up(B * N * sizeof(double));
    w.mail = off; off += round_up(lccrf::pair_mail_words((int)B) * sizeof(unsigned long long));
    w.failed = off; off += round_up(B * sizeof(int));
    const size_t BC = lccrf::scan_supported((int)T) ? B * ((N + chunk - 1) / chunk) : 0;
    const size_t TP = (size_t)lccrf::scan_padded_tags((int)T);
    w.Pl = off; off += round_up(BC * TP * TP * sizeof(float));
    w.rel = off; off += round_up(BC * TP * sizeof(float));
    w.base = off; off += round_up(BC * sizeof(double));
    w.Fv = off; off += round_up(BC * T * sizeof(float));
    w.OF = off; off += round_up(BC * sizeof(double));
    w.Gv = off; off += round_up(BC * T * sizeof(float));
    w.OG = off; off += round_up(BC * sizeof(double));
    const size_t C = (N + chunk - 1) / chunk;
    const size_t gs = BC ? (size_t)lccrf::scan_group_size((int)C) : 0;
    const size_t BG = gs ? B * ((C + gs - 1) / gs) : 0;
    w.Pl2 = off; off += round_up(BG * TP * TP * sizeof(float));
    w.rel2 = off; off += round_up(BG * TP * sizeof(float));
    w.base2 = off; off += round_up(BG * sizeof(double));
    w.Fv2 = off; off += round_up(BG * T * sizeof(float));
    w.OF2 = off; off += round_up(BG * sizeof(double));
    w.Gv2 = off; off += round_up(BG * T * sizeof(float));
    w.OG2 = off; off += round_up(BG * sizeof(double));
    w.lz64 = off; off += round_up(B * sizeof(double));
    w.ha = off; off += round_up(B * T * sizeof(float));
    w.hb = off; off += round_up(B * T * sizeof(float));
    w.hoff = off; off += round_up(B * 2 * sizeof(double));
    w.ent = off; off += round_up(BC * 2 * sizeof(float));
    w.lzf = off; off += round_up(B * sizeof(float));
    w.maps = off; off += round_up(B * N * T);
    w.winmaps = off; off += round_up(lccrf::sample_winmap_bytes((int)B, (int)N, (int)T));
    w.total = off;
    return w;
}
struct MaxWorkspace {
    size_t bp, mid;
    size_t Mx, K, pin;  // chunked scan (T <= 32 only, else empty)
    size_t Mx2, K2, pin2;  // its group level (many chunks only, else empty)
    size_t total;
};
inline MaxWorkspace max_workspace(size_t B, size_t N, size_t T) {
    MaxWorkspace w;
    size_t off = 0;
    const size_t chunk = (size_t)scan_chunk_max((long long)B, (long long)N, (long long)T);
    w.bp = off; off += round_up(B * N * T);
    const size_t BC = lccrf::scan_supported_max((int)T) ? B * ((N + chunk - 1) / chunk) : 0;
    w.mid = off; off += round_up((BC > B ? BC : B) * 2 * T * sizeof(double));
    const size_t TPm = (size_t)lccrf::scan_padded_tags_max((int)T);
    w.Mx = off; off += round_up(BC * TPm * TPm * sizeof(double));
    w.K = off; off += round_up(BC * TPm);
    w.pin = off; off += round_up(BC * sizeof(int32_t));
    const size_t C = (N + chunk - 1) / chunk;
    const size_t gs = BC ? (size_t)lccrf::scan_group_size((int)C) : 0;
    const size_t BG = gs ? B * ((C + gs - 1) / gs) : 0;
    w.Mx2 = off; off += round_up(BG * TPm * TPm * sizeof(double));
    w.K2 = off; off += round_up(BG * TPm);
    w.pin2 = off; off += round_up(BG * sizeof(int32_t));
    w.total = off;
    return w;
}

inline bool shape_ok(int B, int N, int T) {
    if (B < 1 || N < 1 || T < 1 || T > LCCRF_MAX_T) return false;
    const double pots = (double)B * (double)N * (double)T * (double)T;
    // launches use up to 2 * B * ceil(N / 4) workgroups in a 32-bit grid dimension
    return pots < 4.0e18 && (double)B * (double)N < 2.0e9;
}
inline bool dtype_ok(int dt) { return dt == LCCRF_F32 || dt == LCCRF_BF16; }
inline bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

lccrf::ScanGroupBuffers group_buffers(const SumWorkspace& w, char* base) {
    return {reinterpret_cast<float*>(base + w.Pl2), reinterpret_cast<float*>(base + w.rel2),
            reinterpret_cast<double*>(base + w.base2), reinterpret_cast<float*>(base + w.Fv2),
            reinterpret_cast<double*>(base + w.OF2), reinterpret_cast<float*>(base + w.Gv2),
            reinterpret_cast<double*>(base + w.OG2)};
}

int check_common(const void* phi, int dt, int B, int N, int T, const void* ws, size_t ws_bytes, size_t need,
                 int algo) {
    if (!shape_ok(B, N, T) || !dtype_ok(dt)) return LCCRF_EINVAL;
    if (algo < LCCRF_ALGO_AUTO || algo > LCCRF_ALGO_SEQUENTIAL_LANES) return LCCRF_EINVAL;
    if (!phi) return LCCRF_ENULL;
    if (!ws || ws_bytes < need) return LCCRF_EWORKSPACE;
    if (!aligned_to(phi, 16) || !aligned_to(ws, kAlign)) return LCCRF_EALIGN;
    return LCCRF_OK;
}

// Whether LCCRF_ALGO_AUTO takes the chunked scan: the tag set fits its kernels, the chains are long
// enough for the serial depth to dominate (eight chunks; with the chunk chosen by shape that is 64
// positions in small batches), and the batch alone would not fill the chip.  Measured, sum queries:
// with up to 16 tags the sequential schedule costs about 0.3 to 0.6 us a position of the longest
// chain whatever the batch (up to a few waves per SIMD), the scan some 15 us plus 1 ns a position of
// the whole batch, which cross near 450 sequences; with 17 .. 32 tags a chunk product costs eight
// times the matrix instructions and the scan wins up to about 32768 positions a batch (the paper's
// own benchmark size, 128 x 256, is the limit).
//
// Long chains pay whatever the batch holds, as long as the batch is small: the sequential schedule's time grows
// with the length of the longest chain, the scan's with the positions of the whole batch.  Measured, log-partition
// (us; one-wave or four-wave kernels / scan): 17 .. 32 tags 0.26 N / 30 + 0.0016 B N (B=4 N=16384 T=32 4257 / 164,
// B=64 N=2048 549 / 236, B=128 N=1024 280 / 225); 33 .. 48 tags 0.36 N / 30 + 0.0075 B N (B=8 N=4096 T=48
// 1491 / 293, B=32 N=1024 387 / 277); 49 .. 64 tags 0.37 N / 45 + 0.013 B N (B=16 N=1024 T=64 385 / 258).
inline bool scan_pays_sum(int B, int N, int T) {
    if (!lccrf::scan_supported(T) || N < 8 * scan_chunk(B, N, T)) return false;
    if (T <= 16) return B <= 448;
    const double n = (double)N, pb = (double)B;
    // 33 .. 64 tags: a position of a chunk product costs a compute unit about 2.4 us (36 to 64 matrix
    // instructions a wave beside as many exponentials), which the shorter chains pay back up to about 8192
    // positions a batch (B=32, N=256, T=48: marginals 285 -> 124 us; B=128, N=128, T=48: 148 -> 206 us).
    if (T > 48) return (long long)B * N <= 8192 || n * (0.37 - 0.013 * pb) > 45.0;
    if (T > 32) return (long long)B * N <= 8192 || n * (0.36 - 0.0075 * pb) > 30.0;
    return (long long)B * N <= 32768 || n * (0.26 - 0.0016 * pb) > 30.0;
}
// The max-plus scan (16 tags at most) pays its chunk products in double-precision vector
// instructions: it takes chains twice as long to pay, and at most 65536 positions a batch
// (B=256, N=256: 86 us against 62 sequential; B=128, N=512: 87 against 114).
// Longer chains pay in larger batches too: the one-wave kernels take about 0.2 us a position of the longest chain,
// the scan 40 us + 0.75 ns a position of the batch (B=32 N=4096 805 / 140, B=16 N=16384 3193 / 239).
inline bool scan_pays_max(int B, int N, int T) {
    if (!lccrf::scan_supported_max(T) || N < 16 * scan_chunk_max(B, N, T)) return false;
    // 17 .. 32 tags: a chunk product is 32768 additions and maxima in double precision a position; the scan takes
    // about 100 us + 4.5 ns a position of the batch against 0.33 us a position of the longest chain for the one-wave
    // kernels (B=8 N=4096 T=32 1358 / 236, B=4 N=16384 5391 / 401)
    if (T > 16) return (double)N * (0.33 - 0.0045 * B) > 100.0;
    return (long long)B * N <= 65536 || (double)N * (0.195 - 0.00075 * B) > 40.0;
}
// The entropy-like queries make two passes under the scan against one sequential pass: with 17 .. 32
// tags it takes chains twice as long to pay.
// (Long chains at 17 .. 32 tags: one sequential pass 0.43 us a position of the longest chain, the scan's two about
// 20 us + 3 ns a position of the batch: B=64 N=1024 T=24 437 us sequential, B=64 N=2048 T=32 396 under the scan.)
inline bool scan_pays_entropy(int B, int N, int T) {
    if (T > 32 || !lccrf::scan_supported(T)) return false;
    if (T <= 16) return scan_pays_sum(B, N, T);
    if (N < 16 * scan_chunk(B, N, T)) return false;
    return (long long)B * N <= 32768 || (double)N * (0.42 - 0.003 * B) > 30.0;
}
// Sampling under the scan runs every chunk's forward chain with the one-wave kernels (32 tags at most).
// (Long chains at 17 .. 32 tags: 0.7 us a position of the longest chain sequentially, 30 us + 4 ns a position of
// the batch under the scan: B=128 N=1024 T=32 767 us sequential, B=64 N=2048 510 under the scan.)
inline bool scan_pays_sample(int B, int N, int T) {
    if (T > 32 || !lccrf::scan_supported(T)) return false;
    if (T <= 16) return scan_pays_sum(B, N, T);
    if (N < 8 * scan_chunk(B, N, T)) return false;
    return (long long)B * N <= 32768 || (double)N * (0.7 - 0.004 * B) > 30.0;
}

// Whether LCCRF_ALGO_AUTO takes the chain-wave / producer-wave kernels (lccrf_lane.hip) for a sum query
// (op 0: log-partition, 1: marginals).  Their time is set by the serial depth alone, about 12 us plus 0.35 us
// a position at 17 .. 32 tags (0.45 .. 0.6 us at 33 .. 48), as long as every half chain has a compute unit to
// itself; the one-wave and four-wave kernels take 0.7 .. 0.9 us a position, the scan some 30 us plus 2.9 ns a
// position of the whole batch at 17 .. 32 tags.  Measured (marginals, us; lanes / scan / sequential):
// B=128 N=256 T=32 102 / 122 / 197, B=256 N=256 T=32 168 / 246 / 227, B=32 N=64 T=32 38 / 40 / 57,
// B=32 N=256 T=32 98 / 61 / 193, B=128 N=128 T=48 92 / 216 / 133, B=64 N=64 T=48 47 / 78 / 73.  Above 48 tags the
// second pass does not pay (its producers spill), the first still does (B=32 N=256 T=64 log-partition 76 / 121 / 108).
// With 8 .. 16 tags they take about 15.5 us plus 0.24 us a position, up to one sequence a compute unit (two
// workgroups of twelve waves each), against 11 us plus 0.6 us a position for the one-wave kernels and some 27 us plus
// 0.75 ns a position of the whole batch for the scan (marginals, lanes / scan / sequential: B=128 N=32 T=13
// 23 / - / 32, B=256 N=128 T=16 50 / 53 / 98, B=128 N=128 T=9 46 / 41 / 99, B=32 N=256 T=8 75 / 38 / 170,
// B=512 N=64 T=16 62 / - / 55).
inline bool lanes_pay_sum(int op, int B, int N, int T) {
    if (!lccrf::lane_chains_supported(T)) return false;
    const int cus = current_device_cus();
    if (T <= 16) {
        if (B > cus || N < 16) return false;
        return !scan_pays_sum(B, N, T) || (double)N * (0.24 - 0.00075 * B) < 10.0;
    }
    // Against the scan, where it would be taken (us, log-partition / marginals; these kernels and the scan):
    // 17 .. 32 tags 15 + 0.124 N / 20 + 0.257 N and 30 + 0.0016 B N / 40 + 0.0035 B N (B=16 N=4096 T=32 521 / 1054
    // and 139 / 271, B=64 N=1024 144 / 282 and 128 / 259, B=128 N=1024 146 / 343 and 225 / 483);
    // 33 .. 48 tags 15 + 0.18 N / 20 + 0.41 N and 30 + 0.0075 B N / 100 + 0.0107 B N (B=16 N=2048 T=48 379 / 858
    // and 283 / 471, B=32 N=1024 200 / 449 and 277 / 453); 49 .. 64 tags, log-partition, 15 + 0.2 N and
    // 45 + 0.013 B N (B=16 N=1024 T=64 218 and 258).
    const double n = (double)N;
    if (T <= 32) {
        if (B > cus) return false;
        if (!scan_pays_sum(B, N, T)) return true;
        return op == 0 ? n * (0.124 - 0.0016 * B) < 15.0 : n * (0.257 - 0.0035 * B) < 20.0;
    }
    if (2 * B > cus || (T > 48 && op != 0)) return false;
    if (!scan_pays_sum(B, N, T)) return true;
    if (T > 48) return n * (0.2 - 0.013 * B) < 30.0;
    return op == 0 ? n * (0.18 - 0.0075 * B) < 15.0 : n * (0.41 - 0.0107 * B) < 80.0;
}

// Whether LCCRF_ALGO_AUTO gives the max-plus chains to the chain-wave kernels (lccrf_lane_max.hip) rather than to
// the one-wave / four-wave kernels.  They pay while every workgroup (two a sequence, eight waves each) is resident
// at once: four a compute unit up to 16 tags, two up to 32, one up to 48 (their LDS rings).  Measured, whole
// argmax, sequential / these (us): B=256 N=256 T=16 71 / 45, B=512 N=256 T=16 79 / 62, B=1024 N=64 T=16 33 / 38;
// B=128 N=256 T=32 106 / 59, B=256 N=128 T=32 64 / 57, B=384 N=128 T=32 68 / 75; B=128 N=128 T=48 99 / 74,
// B=64 N=256 T=40 181 / 117, B=256 N=128 T=48 127 / 130; above 48 tags the ring holds too few matrices
// (B=32 N=256 T=64 182 / 208).  Tag counts that are no multiple of four gain the same (B=128 N=128 T=45 106 / 76,
// T=48 96 / 72; B=32 N=64 T=30 43 / 27); chains of fewer than 16 positions do not pay the kernel's start
// (B=4 N=8 T=5 17.8 / 18.6).
inline bool lanes_pay_max(int B, int N, int T) {
    if (!lccrf::lane_max_supported(T) || T > 48 || N < 16) return false;
    const int cus = current_device_cus();
    return T <= 16 ? B <= 2 * cus : T <= 32 ? B <= cus : 2 * B <= cus;
}
// Whether AUTO takes the max-plus scan: where it would pay against the one-wave kernels, unless the chain-wave
// kernels are quicker still (up to 16 tags they take about 16 us + 0.084 us a position whatever the batch, the
// scan about 40 us + 0.75 ns a position of the batch: B=64 N=512 59 / 61, B=64 N=768 80 / 74, B=8 N=512 58 / 45,
// B=128 N=512 61 / 76, B=256 N=256 41 / 75, B=128 N=2048 190 / 254, B=64 N=4096 358 / 237, B=16 N=16384 1368 / 239).
inline bool scan_taken_max(int B, int N, int T) {
    if (!scan_pays_max(B, N, T)) return false;
    // (17 .. 32 tags: the chain-wave kernels take 15 us + 0.133 us a position: B=8 N=4096 T=32 560 / 236,
    // B=16 N=512 83 / 114, B=32 N=1024 153 / 212, B=1 N=8192 1098 / 189)
    if (T > 16) return !(lanes_pay_max(B, N, T) && (double)N * (0.133 - 0.0045 * B) <= 85.0);
    return !(lanes_pay_max(B, N, T) && (double)N * (0.084 - 0.00075 * B) < 24.0);
}

int sum_query(int op, const void* phi, int dt, const int32_t* lengths, int B, int N, int T, float* logZ,
              float* marginals, void* workspace, size_t workspace_bytes, void* stream, int algo,
              void* ev_begin = nullptr, void* ev_between = nullptr, void* ev_end = nullptr) {
    const size_t need = lccrf_workspace_bytes(op == 0 ? LCCRF_OP_LOGZ : LCCRF_OP_MARGINALS, B, N, T,
                                              (lccrf_dtype)dt);
    const int rc = check_common(phi, dt, B, N, T, workspace, workspace_bytes, need, algo);
    if (rc != LCCRF_OK) return rc;
    if (op == 0 && !logZ) return LCCRF_ENULL;
    if (op == 1 && !marginals) return LCCRF_ENULL;
    if ((logZ && !aligned_to(logZ, 4)) || (marginals && !aligned_to(marginals, 16))) return LCCRF_EALIGN;
    if (lengths && !aligned_to(lengths, 4)) return LCCRF_EALIGN;
    if (algo == LCCRF_ALGO_SCAN && !lccrf::scan_supported(T)) return LCCRF_ENOTIMPL;
    if (algo == LCCRF_ALGO_SEQUENTIAL_LANES && !lccrf::lane_chains_supported(T)) return LCCRF_ENOTIMPL;
    const bool lanes = algo == LCCRF_ALGO_SEQUENTIAL_LANES || (algo == LCCRF_ALGO_AUTO && lanes_pay_sum(op, B, N, T));
    const SumWorkspace w = sum_workspace(B, N, T);
    char* base = static_cast<char*>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (ev_begin && hipEventRecord(static_cast<hipEvent_t>(ev_begin), st) != hipSuccess) return LCCRF_ELAUNCH;
    if (algo == LCCRF_ALGO_SCAN || (algo == LCCRF_ALGO_AUTO && !lanes && scan_pays_sum(B, N, T))) {
        float* Fv = reinterpret_cast<float*>(base + w.Fv);
        double* OF = reinterpret_cast<double*>(base + w.OF);
        float* Gv = reinterpret_cast<float*>(base + w.Gv);
        double* OG = reinterpret_cast<double*>(base + w.OG);
        hipError_t e = lccrf::launch_scan_boundaries(dt, phi, lengths, B, N, T, scan_chunk(B, N, T),
                                                     reinterpret_cast<float*>(base + w.Pl),
                                                     reinterpret_cast<float*>(base + w.rel),
                                                     reinterpret_cast<double*>(base + w.base), Fv, OF, Gv, OG,
                                                     group_buffers(w, base), logZ, op == 1, st);
        if (e == hipSuccess && op == 1)
            e = lccrf::launch_chunked_marginals(dt, phi, lengths, B, N, T, reinterpret_cast<float*>(base + w.ua),
                                                reinterpret_cast<float*>(base + w.ub),
                                                reinterpret_cast<double*>(base + w.Oa),
                                                reinterpret_cast<double*>(base + w.Ob), marginals, scan_chunk(B, N, T), Fv,
                                                OF, Gv, OG, st, static_cast<hipEvent_t>(ev_between), false);
        if (e != hipSuccess) return LCCRF_ELAUNCH;
        if (ev_end && hipEventRecord(static_cast<hipEvent_t>(ev_end), st) != hipSuccess) return LCCRF_ELAUNCH;
        return LCCRF_OK;
    }
    const hipError_t e = lccrf::launch_sequential_sum(
        op, dt, phi, lengths, B, N, T, reinterpret_cast<float*>(base + w.ua), reinterpret_cast<float*>(base + w.ub),
        reinterpret_cast<double*>(base + w.Oa), reinterpret_cast<double*>(base + w.Ob), logZ, marginals, st,
        static_cast<hipEvent_t>(ev_between), algo == LCCRF_ALGO_SEQUENTIAL_EXACT,
        algo == LCCRF_ALGO_AUTO ? reinterpret_cast<unsigned long long*>(base + w.mail) : nullptr,
        reinterpret_cast<int*>(base + w.failed), nullptr, nullptr, nullptr,
        g_pair_poll_limit.load(std::memory_order_relaxed), algo == LCCRF_ALGO_AUTO ? current_device_cus() : 0, lanes,
        g_lane_poll_limit.load(std::memory_order_relaxed));
    if (e != hipSuccess) return LCCRF_ELAUNCH;
    if (ev_end && hipEventRecord(static_cast<hipEvent_t>(ev_end), st) != hipSuccess) return LCCRF_ELAUNCH;
    return LCCRF_OK;
}

}  // namespace

extern "C" {

size_t lccrf_workspace_bytes(lccrf_op op, int B, int N, int T, lccrf_dtype dt) {
    const KnobSnapshot knobs;
    if (!shape_ok(B, N, T) || !dtype_ok(dt)) return 0;
    switch (op) {
        case LCCRF_OP_LOGZ:
        case LCCRF_OP_MARGINALS:
        case LCCRF_OP_LOG_PROB:
        case LCCRF_OP_ENTROPY:
        case LCCRF_OP_SAMPLE:
        case LCCRF_OP_CROSS_ENTROPY: return sum_workspace(B, N, T).total;
        case LCCRF_OP_ARGMAX: return max_workspace(B, N, T).total;
        default: return 0;
    }
}

int lccrf_auto_algo(lccrf_op op, int B, int N, int T) {
    const KnobSnapshot knobs;
    if (!shape_ok(B, N, T)) return LCCRF_EINVAL;
    bool scan;
    switch (op) {
        case LCCRF_OP_LOGZ:
        case LCCRF_OP_MARGINALS:
            if (lanes_pay_sum(op == LCCRF_OP_LOGZ ? 0 : 1, B, N, T)) return LCCRF_ALGO_SEQUENTIAL_LANES;
            scan = scan_pays_sum(B, N, T);
            break;
        case LCCRF_OP_LOG_PROB: scan = scan_pays_sum(B, N, T); break;
        case LCCRF_OP_SAMPLE: scan = scan_pays_sample(B, N, T); break;
        case LCCRF_OP_ARGMAX:
            scan = scan_taken_max(B, N, T);
            if (!scan && lanes_pay_max(B, N, T)) return LCCRF_ALGO_SEQUENTIAL_LANES;
            break;
        case LCCRF_OP_ENTROPY:
        case LCCRF_OP_CROSS_ENTROPY: scan = scan_pays_entropy(B, N, T); break;
        default: return LCCRF_EINVAL;
    }
    return scan ? LCCRF_ALGO_SCAN : LCCRF_ALGO_SEQUENTIAL;
}

int lccrf_log_partition_algo(const void* phi, lccrf_dtype dt, const int32_t* lengths, int B, int N, int T,
                             float* logZ, void* workspace, size_t workspace_bytes, void* stream, lccrf_algo algo) {
    const KnobSnapshot knobs;
    return sum_query(0, phi, dt, lengths, B, N, T, logZ, nullptr, workspace, workspace_bytes, stream, algo);
}

int lccrf_marginals_algo(const void* phi, lccrf_dtype dt, const int32_t* lengths, int B, int N, int T, float* logZ,
                         float* marginals, void* workspace, size_t workspace_bytes, void* stream, lccrf_algo algo) {
    const KnobSnapshot knobs;
    return sum_query(1, phi, dt, lengths, B, N, T, logZ, marginals, workspace, workspace_bytes, stream, algo);
}

int lccrf_marginals_timed(const void* phi, lccrf_dtype dt, const int32_t* lengths, int B, int N, int T, float* logZ,
                          float* marginals, void* workspace, size_t workspace_bytes, void* stream, lccrf_algo algo,
                          void* ev_begin, void* ev_between, void* ev_end) {
    const KnobSnapshot knobs;
    return sum_query(1, phi, dt, lengths, B, N, T, logZ, marginals, workspace, workspace_bytes, stream, algo,
                     ev_begin, ev_between, ev_end);
}

int lccrf_argmax_algo(const void* phi, lccrf_dtype dt, const int32_t* lengths, int B, int N, int T,
                      float* best_score, int32_t* tags, void* workspace, size_t workspace_bytes, void* stream,
                      lccrf_algo algo) {
    const KnobSnapshot knobs;
    const size_t need = lccrf_workspace_bytes(LCCRF_OP_ARGMAX, B, N, T, dt);
    const int rc = check_common(phi, dt, B, N, T, workspace, workspace_bytes, need, algo);
    if (rc != LCCRF_OK) return rc;
    if (!tags) return LCCRF_ENULL;
    if (!aligned_to(tags, 4) || (best_score && !aligned_to(best_score, 4))) return LCCRF_EALIGN;
    if (lengths && !aligned_to(lengths, 4)) return LCCRF_EALIGN;
    if (algo == LCCRF_ALGO_SCAN && !lccrf::scan_supported_max(T)) return LCCRF_ENOTIMPL;
    if (algo == LCCRF_ALGO_SEQUENTIAL_LANES && !lccrf::lane_max_supported(T)) return LCCRF_ENOTIMPL;
    const MaxWorkspace w = max_workspace(B, N, T);
    char* base = static_cast<char*>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t* bp = reinterpret_cast<uint8_t*>(base + w.bp);
    double* mid = reinterpret_cast<double*>(base + w.mid);
    hipError_t e;
    if (algo == LCCRF_ALGO_SCAN || (algo == LCCRF_ALGO_AUTO && scan_taken_max(B, N, T))) {
        int32_t* pin = reinterpret_cast<int32_t*>(base + w.pin);
        e = lccrf::launch_scan_pins(dt, phi, lengths, B, N, T, scan_chunk_max(B, N, T), reinterpret_cast<double*>(base + w.Mx),
                                    reinterpret_cast<uint8_t*>(base + w.K), pin,
                                    {reinterpret_cast<double*>(base + w.Mx2), reinterpret_cast<uint8_t*>(base + w.K2),
                                     reinterpret_cast<int32_t*>(base + w.pin2)},
                                    best_score, st);
        if (e == hipSuccess)
            e = lccrf::launch_chunked_max(dt, phi, lengths, B, N, T, bp, mid, tags, scan_chunk_max(B, N, T), pin, st);
    } else {
        const bool lanes = algo == LCCRF_ALGO_SEQUENTIAL_LANES || (algo == LCCRF_ALGO_AUTO && lanes_pay_max(B, N, T));
        e = lccrf::launch_sequential_max(dt, phi, lengths, B, N, T, bp, mid, best_score, tags, st, lanes,
                                         g_lane_poll_limit.load(std::memory_order_relaxed));
    }
    return e == hipSuccess ? LCCRF_OK : LCCRF_ELAUNCH;
}

int lccrf_log_partition(const void* phi, lccrf_dtype dt, const int32_t* lengths, int B, int N, int T, float* logZ,
                        void* workspace, size_t workspace_bytes, void* stream) {
    return lccrf_log_partition_algo(phi, dt, lengths, B, N, T, logZ, workspace, workspace_bytes, stream,
                                    LCCRF_ALGO_AUTO);
}

int lccrf_marginals(const void* phi, lccrf_dtype dt, const int32_t* lengths, int B, int N, int T, float* logZ,
                    float* marginals, void* workspace, size_t workspace_bytes, void* stream) {
    return lccrf_marginals_algo(phi, dt, lengths, B, N, T, logZ, marginals, workspace, workspace_bytes, stream,
                                LCCRF_ALGO_AUTO);
}

size_t lccrf_static_scratch_bytes(void) { return LCCRF_STATIC_SCRATCH_BYTES; }

int lccrf_marginals_static(const void* phi, lccrf_dtype dt, const int32_t* lengths, int B, int N, int T, float* logZ,
                           float* marginals, void* stream) {
    const KnobSnapshot knobs;
    const size_t need = lccrf_workspace_bytes(LCCRF_OP_MARGINALS, B, N, T, dt);
    if (need == 0) return LCCRF_EINVAL;
    if (need > LCCRF_STATIC_SCRATCH_BYTES) return LCCRF_ETOOBIG;
    if (!phi || !marginals) return LCCRF_ENULL;
    void* ws = static_scratch();
    if (!ws) return LCCRF_ELAUNCH;
    return lccrf_marginals_algo(phi, dt, lengths, B, N, T, logZ, marginals, ws, LCCRF_STATIC_SCRATCH_BYTES, stream,
                                LCCRF_ALGO_AUTO);
}

int lccrf_argmax(const void* phi, lccrf_dtype dt, const int32_t* lengths, int B, int N, int T, float* best_score,
                 int32_t* tags, void* workspace, size_t workspace_bytes, void* stream) {
    return lccrf_argmax_algo(phi, dt, lengths, B, N, T, best_score, tags, workspace, workspace_bytes, stream,
                             LCCRF_ALGO_AUTO);
}

// log Z [B] in double precision into the workspace's lz64 slot, by the schedule AUTO would take.
static hipError_t launch_log_partition64(const void* phi, int dt, const int32_t* lengths, int B, int N, int T,
                                         const SumWorkspace& w, char* base, hipStream_t st) {
    double* lz64 = reinterpret_cast<double*>(base + w.lz64);
    if (scan_pays_sum(B, N, T))
        return lccrf::launch_scan_boundaries(
            dt, phi, lengths, B, N, T, scan_chunk(B, N, T), reinterpret_cast<float*>(base + w.Pl),
            reinterpret_cast<float*>(base + w.rel), reinterpret_cast<double*>(base + w.base),
            reinterpret_cast<float*>(base + w.Fv), reinterpret_cast<double*>(base + w.OF),
            reinterpret_cast<float*>(base + w.Gv), reinterpret_cast<double*>(base + w.OG), group_buffers(w, base),
            nullptr, false, st, lz64);
    return lccrf::launch_sequential_sum(0, dt, phi, lengths, B, N, T, reinterpret_cast<float*>(base + w.ua),
                                        reinterpret_cast<float*>(base + w.ub), reinterpret_cast<double*>(base + w.Oa),
                                        reinterpret_cast<double*>(base + w.Ob), nullptr, nullptr, st, nullptr, false,
                                        nullptr, nullptr, lz64);
}

int lccrf_log_prob(const void* phi, lccrf_dtype dt, const int32_t* lengths, const int32_t* tags, int B, int N, int T,
                   float* log_prob, void* workspace, size_t workspace_bytes, void* stream) {
    const KnobSnapshot knobs;
    const size_t need = lccrf_workspace_bytes(LCCRF_OP_LOG_PROB, B, N, T, dt);
    const int rc = check_common(phi, dt, B, N, T, workspace, workspace_bytes, need, LCCRF_ALGO_AUTO);
    if (rc != LCCRF_OK) return rc;
    if (!tags || !log_prob) return LCCRF_ENULL;
    if (!aligned_to(tags, 4) || !aligned_to(log_prob, 4) || (lengths && !aligned_to(lengths, 4))) return LCCRF_EALIGN;
    const SumWorkspace w = sum_workspace(B, N, T);
    char* base = static_cast<char*>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    double* lz64 = reinterpret_cast<double*>(base + w.lz64);
    hipError_t e = launch_log_partition64(phi, dt, lengths, B, N, T, w, base, st);
    if (e == hipSuccess) e = lccrf::launch_path_log_prob(dt, phi, lengths, tags, B, N, T, lz64, log_prob, st);
    return e == hipSuccess ? LCCRF_OK : LCCRF_ELAUNCH;
}

int lccrf_entropy(const void* phi, lccrf_dtype dt, const int32_t* lengths, int B, int N, int T, float* entropy,
                  void* workspace, size_t workspace_bytes, void* stream) {
    const KnobSnapshot knobs;
    const size_t need = lccrf_workspace_bytes(LCCRF_OP_ENTROPY, B, N, T, dt);
    const int rc = check_common(phi, dt, B, N, T, workspace, workspace_bytes, need, LCCRF_ALGO_AUTO);
    if (rc != LCCRF_OK) return rc;
    if (!entropy) return LCCRF_ENULL;
    if (!aligned_to(entropy, 4) || (lengths && !aligned_to(lengths, 4))) return LCCRF_EALIGN;
    const SumWorkspace w = sum_workspace(B, N, T);
    char* base = static_cast<char*>(workspace);
    if (scan_pays_entropy(B, N, T)) {
        // Under the chunked scan a chain cannot carry its conditional entropy across chunks; the second pass
        // adds up the entropy edge by edge instead, H = H(y_0) + sum_i H(y_i | y_{i-1}), from the marginals
        // it forms in registers.
        hipStream_t st = static_cast<hipStream_t>(stream);
        float* Fv = reinterpret_cast<float*>(base + w.Fv);
        double* OF = reinterpret_cast<double*>(base + w.OF);
        float* Gv = reinterpret_cast<float*>(base + w.Gv);
        double* OG = reinterpret_cast<double*>(base + w.OG);
        float* ent = reinterpret_cast<float*>(base + w.ent);
        float* lzf = reinterpret_cast<float*>(base + w.lzf);
        hipError_t e = lccrf::launch_scan_boundaries(dt, phi, lengths, B, N, T, scan_chunk(B, N, T),
                                                     reinterpret_cast<float*>(base + w.Pl),
                                                     reinterpret_cast<float*>(base + w.rel),
                                                     reinterpret_cast<double*>(base + w.base), Fv, OF, Gv, OG,
                                                     group_buffers(w, base), lzf, true, st);
        if (e == hipSuccess)
            e = lccrf::launch_chunked_marginals(dt, phi, lengths, B, N, T, reinterpret_cast<float*>(base + w.ua),
                                                reinterpret_cast<float*>(base + w.ub),
                                                reinterpret_cast<double*>(base + w.Oa),
                                                reinterpret_cast<double*>(base + w.Ob), nullptr, scan_chunk(B, N, T), Fv, OF,
                                                Gv, OG, st, nullptr, false, ent);
        if (e == hipSuccess) e = lccrf::launch_entropy_reduce(ent, lengths, lzf, B, N, scan_chunk(B, N, T), entropy, st);
        return e == hipSuccess ? LCCRF_OK : LCCRF_ELAUNCH;
    }
    const hipError_t e = lccrf::launch_entropy(
        dt, phi, lengths, B, N, T, reinterpret_cast<float*>(base + w.ua), reinterpret_cast<float*>(base + w.ub),
        reinterpret_cast<double*>(base + w.Oa), reinterpret_cast<double*>(base + w.Ob),
        reinterpret_cast<float*>(base + w.ha), reinterpret_cast<float*>(base + w.hb), entropy,
        static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LCCRF_OK : LCCRF_ELAUNCH;
}

static int cross_query(bool kl, const void* phi_p, const void* phi_q, lccrf_dtype dt, const int32_t* lengths, int B, int N,
                       int T, float* out, void* workspace, size_t workspace_bytes, void* stream) {
    const KnobSnapshot knobs;
    const size_t need = lccrf_workspace_bytes(LCCRF_OP_CROSS_ENTROPY, B, N, T, dt);
    const int rc = check_common(phi_p, dt, B, N, T, workspace, workspace_bytes, need, LCCRF_ALGO_AUTO);
    if (rc != LCCRF_OK) return rc;
    if (!phi_q || !out) return LCCRF_ENULL;
    if (!aligned_to(phi_q, 16) || !aligned_to(out, 4) || (lengths && !aligned_to(lengths, 4))) return LCCRF_EALIGN;
    const SumWorkspace w = sum_workspace(B, N, T);
    char* base = static_cast<char*>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    // log Z_q first: the chains of p then reuse the vectors' storage, the double-precision result stays
    hipError_t e = launch_log_partition64(phi_q, dt, lengths, B, N, T, w, base, st);
    if (scan_pays_entropy(B, N, T)) {
        // Long chains over few tags: the chains of p under the chunked scan, as for the entropy; the second
        // pass adds up the expectation of phi_q (of phi_q - phi_p) edge by edge from the marginals of p it
        // forms in registers.
        float* Fv = reinterpret_cast<float*>(base + w.Fv);
        double* OF = reinterpret_cast<double*>(base + w.OF);
        float* Gv = reinterpret_cast<float*>(base + w.Gv);
        double* OG = reinterpret_cast<double*>(base + w.OG);
        float* ent = reinterpret_cast<float*>(base + w.ent);
        double* lzp = reinterpret_cast<double*>(base + w.hoff);
        if (e == hipSuccess)
            e = lccrf::launch_scan_boundaries(dt, phi_p, lengths, B, N, T, scan_chunk(B, N, T),
                                              reinterpret_cast<float*>(base + w.Pl), reinterpret_cast<float*>(base + w.rel),
                                              reinterpret_cast<double*>(base + w.base), Fv, OF, Gv, OG,
                                              group_buffers(w, base), nullptr, true, st, lzp);
        if (e == hipSuccess)
            e = lccrf::launch_chunked_marginals(dt, phi_p, lengths, B, N, T, reinterpret_cast<float*>(base + w.ua),
                                                reinterpret_cast<float*>(base + w.ub),
                                                reinterpret_cast<double*>(base + w.Oa),
                                                reinterpret_cast<double*>(base + w.Ob), nullptr, scan_chunk(B, N, T), Fv, OF,
                                                Gv, OG, st, nullptr, false, ent, phi_q, kl);
        if (e == hipSuccess)
            e = lccrf::launch_cross_reduce(kl, ent, lengths, reinterpret_cast<const double*>(base + w.lz64), lzp, B, N,
                                           scan_chunk(B, N, T), out, st);
        return e == hipSuccess ? LCCRF_OK : LCCRF_ELAUNCH;
    }
    if (e == hipSuccess)
        e = lccrf::launch_cross(kl, dt, phi_p, phi_q, lengths, B, N, T, reinterpret_cast<float*>(base + w.ua),
                                reinterpret_cast<float*>(base + w.ub), reinterpret_cast<double*>(base + w.Oa),
                                reinterpret_cast<double*>(base + w.Ob), reinterpret_cast<float*>(base + w.ha),
                                reinterpret_cast<float*>(base + w.hb), reinterpret_cast<double*>(base + w.hoff),
                                reinterpret_cast<const double*>(base + w.lz64), out, st);
    return e == hipSuccess ? LCCRF_OK : LCCRF_ELAUNCH;
}

int lccrf_cross_entropy(const void* phi_p, const void* phi_q, lccrf_dtype dt, const int32_t* lengths, int B, int N, int T,
                        float* out, void* workspace, size_t workspace_bytes, void* stream) {
    return cross_query(false, phi_p, phi_q, dt, lengths, B, N, T, out, workspace, workspace_bytes, stream);
}

int lccrf_kl_divergence(const void* phi_p, const void* phi_q, lccrf_dtype dt, const int32_t* lengths, int B, int N, int T,
                        float* out, void* workspace, size_t workspace_bytes, void* stream) {
    return cross_query(true, phi_p, phi_q, dt, lengths, B, N, T, out, workspace, workspace_bytes, stream);
}

int lccrf_semi_markov_log_partition(const void* phi, lccrf_dtype dt, const int32_t* lengths, int B, int N, int K, int T,
                                    float* logZ, void* stream) {
    if (!shape_ok(B, N, T) || !dtype_ok(dt) || K < 1) return LCCRF_EINVAL;
    if ((double)B * N * K * T * T >= 4.0e18) return LCCRF_EINVAL;
    if (!phi || !logZ) return LCCRF_ENULL;
    if (!aligned_to(phi, 16) || !aligned_to(logZ, 4) || (lengths && !aligned_to(lengths, 4))) return LCCRF_EALIGN;
    if (!lccrf::semi_markov_supported(K, T)) return LCCRF_ENOTIMPL;
    const hipError_t e = lccrf::launch_semi_markov_forward(dt, phi, lengths, B, N, K, T, logZ, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LCCRF_OK : LCCRF_ELAUNCH;
}

static int sample_query(const void* phi, lccrf_dtype dt, const int32_t* lengths, const float* uniforms, bool seeded,
                        unsigned long long seed, int B, int N, int T, int32_t* tags, void* workspace, size_t workspace_bytes,
                        void* stream) {
    const KnobSnapshot knobs;
    const size_t need = lccrf_workspace_bytes(LCCRF_OP_SAMPLE, B, N, T, dt);
    const int rc = check_common(phi, dt, B, N, T, workspace, workspace_bytes, need, LCCRF_ALGO_AUTO);
    if (rc != LCCRF_OK) return rc;
    if ((!seeded && !uniforms) || !tags) return LCCRF_ENULL;
    if ((uniforms && !aligned_to(uniforms, 4)) || !aligned_to(tags, 4) || (lengths && !aligned_to(lengths, 4))) return LCCRF_EALIGN;
    const SumWorkspace w = sum_workspace(B, N, T);
    char* base = static_cast<char*>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    float* ua = reinterpret_cast<float*>(base + w.ua);
    float* ub = reinterpret_cast<float*>(base + w.ub);
    double* Oa = reinterpret_cast<double*>(base + w.Oa);
    double* Ob = reinterpret_cast<double*>(base + w.Ob);
    hipError_t e;
    if (scan_pays_sample(B, N, T)) {  // alpha everywhere, chunk by chunk from the scan's boundary vectors
        float* Fv = reinterpret_cast<float*>(base + w.Fv);
        double* OF = reinterpret_cast<double*>(base + w.OF);
        e = lccrf::launch_scan_boundaries(dt, phi, lengths, B, N, T, scan_chunk(B, N, T), reinterpret_cast<float*>(base + w.Pl),
                                          reinterpret_cast<float*>(base + w.rel), reinterpret_cast<double*>(base + w.base),
                                          Fv, OF, reinterpret_cast<float*>(base + w.Gv),
                                          reinterpret_cast<double*>(base + w.OG), group_buffers(w, base), nullptr, false, st);
        if (e == hipSuccess)
            e = lccrf::launch_chunked_full_forward(dt, phi, lengths, B, N, T, ua, ub, Oa, Ob, scan_chunk(B, N, T), Fv, OF, st);
    } else {
        e = lccrf::launch_full_forward(dt, phi, lengths, B, N, T, ua, ub, Oa, Ob, st);
    }
    if (e == hipSuccess)
        e = lccrf::launch_backward_sample(dt, phi, lengths, ua, Oa, seeded ? nullptr : uniforms, seed, B, N, T,
                                          reinterpret_cast<uint8_t*>(base + w.maps),
                                          reinterpret_cast<uint8_t*>(base + w.winmaps), tags, st);
    return e == hipSuccess ? LCCRF_OK : LCCRF_ELAUNCH;
}

int lccrf_sample(const void* phi, lccrf_dtype dt, const int32_t* lengths, const float* uniforms, int B, int N, int T,
                 int32_t* tags, void* workspace, size_t workspace_bytes, void* stream) {
    return sample_query(phi, dt, lengths, uniforms, false, 0ull, B, N, T, tags, workspace, workspace_bytes, stream);
}

int lccrf_sample_seeded(const void* phi, lccrf_dtype dt, const int32_t* lengths, uint64_t seed, int B, int N, int T,
                        int32_t* tags, void* workspace, size_t workspace_bytes, void* stream) {
    return sample_query(phi, dt, lengths, nullptr, true, (unsigned long long)seed, B, N, T, tags, workspace,
                        workspace_bytes, stream);
}

// Common checks of the structured calls.
static int check_structured(const float* emit, const float* trans, const int32_t* lengths, int B, int N, int T,
                            const void* ws, size_t ws_bytes, size_t need) {
    if (!shape_ok(B, N, T)) return LCCRF_EINVAL;
    if (!emit || !trans) return LCCRF_ENULL;
    if (!ws || ws_bytes < need) return LCCRF_EWORKSPACE;
    if (!aligned_to(emit, 16) || !aligned_to(trans, 16) || !aligned_to(ws, kAlign)) return LCCRF_EALIGN;
    if (lengths && !aligned_to(lengths, 4)) return LCCRF_EALIGN;
    if (!lccrf::structured_supported(T)) return LCCRF_ENOTIMPL;
    return LCCRF_OK;
}

static int structured_sum(int op, const float* emit, const float* trans, const int32_t* lengths, int B, int N, int T,
                          float* logZ, float* marginals, void* workspace, size_t workspace_bytes, void* stream) {
    const KnobSnapshot knobs;
    const size_t need = lccrf_workspace_bytes(op == 0 ? LCCRF_OP_LOGZ : LCCRF_OP_MARGINALS, B, N, T, LCCRF_F32);
    const int rc = check_structured(emit, trans, lengths, B, N, T, workspace, workspace_bytes, need);
    if (rc != LCCRF_OK) return rc;
    if (op == 0 && !logZ) return LCCRF_ENULL;
    if (op == 1 && !marginals) return LCCRF_ENULL;
    if ((logZ && !aligned_to(logZ, 4)) || (marginals && !aligned_to(marginals, 16))) return LCCRF_EALIGN;
    const SumWorkspace w = sum_workspace(B, N, T);
    char* base = static_cast<char*>(workspace);
    // the schedule lccrf_auto_algo reports for the dense call of this shape
    const bool lanes = lanes_pay_sum(op, B, N, T) && T <= 48;  // (above, the transition entries no longer fit a producer's registers)
    if (!lanes && scan_pays_sum(B, N, T)) {
        hipStream_t st = static_cast<hipStream_t>(stream);
        float* Fv = reinterpret_cast<float*>(base + w.Fv);
        double* OF = reinterpret_cast<double*>(base + w.OF);
        float* Gv = reinterpret_cast<float*>(base + w.Gv);
        double* OG = reinterpret_cast<double*>(base + w.OG);
        hipError_t e = lccrf::launch_scan_boundaries(LCCRF_F32, nullptr, lengths, B, N, T, scan_chunk(B, N, T),
                                                     reinterpret_cast<float*>(base + w.Pl),
                                                     reinterpret_cast<float*>(base + w.rel),
                                                     reinterpret_cast<double*>(base + w.base), Fv, OF, Gv, OG,
                                                     group_buffers(w, base), logZ, op == 1, st, nullptr, emit, trans);
        if (e == hipSuccess && op == 1)
            e = lccrf::launch_chunked_marginals(LCCRF_F32, nullptr, lengths, B, N, T,
                                                reinterpret_cast<float*>(base + w.ua),
                                                reinterpret_cast<float*>(base + w.ub),
                                                reinterpret_cast<double*>(base + w.Oa),
                                                reinterpret_cast<double*>(base + w.Ob), marginals, scan_chunk(B, N, T),
                                                Fv, OF, Gv, OG, st, nullptr, false, nullptr, nullptr, false, emit, trans);
        return e == hipSuccess ? LCCRF_OK : LCCRF_ELAUNCH;
    }
    const hipError_t e = lccrf::launch_sequential_sum(
        op, LCCRF_F32, nullptr, lengths, B, N, T, reinterpret_cast<float*>(base + w.ua),
        reinterpret_cast<float*>(base + w.ub), reinterpret_cast<double*>(base + w.Oa),
        reinterpret_cast<double*>(base + w.Ob), logZ, marginals, static_cast<hipStream_t>(stream), nullptr, false,
        nullptr, nullptr, nullptr, emit, trans, 0, 0, lanes, g_lane_poll_limit.load(std::memory_order_relaxed));
    return e == hipSuccess ? LCCRF_OK : LCCRF_ELAUNCH;
}

int lccrf_log_partition_structured(const float* emit, const float* trans, const int32_t* lengths, int B, int N, int T,
                                   float* logZ, void* workspace, size_t workspace_bytes, void* stream) {
    return structured_sum(0, emit, trans, lengths, B, N, T, logZ, nullptr, workspace, workspace_bytes, stream);
}

int lccrf_marginals_structured(const float* emit, const float* trans, const int32_t* lengths, int B, int N, int T,
                               float* logZ, float* marginals, void* workspace, size_t workspace_bytes, void* stream) {
    return structured_sum(1, emit, trans, lengths, B, N, T, logZ, marginals, workspace, workspace_bytes, stream);
}

int lccrf_argmax_structured(const float* emit, const float* trans, const int32_t* lengths, int B, int N, int T,
                            float* best_score, int32_t* tags, void* workspace, size_t workspace_bytes, void* stream) {
    const KnobSnapshot knobs;
    const size_t need = lccrf_workspace_bytes(LCCRF_OP_ARGMAX, B, N, T, LCCRF_F32);
    const int rc = check_structured(emit, trans, lengths, B, N, T, workspace, workspace_bytes, need);
    if (rc != LCCRF_OK) return rc;
    if (!tags) return LCCRF_ENULL;
    if (!aligned_to(tags, 4) || (best_score && !aligned_to(best_score, 4))) return LCCRF_EALIGN;
    const MaxWorkspace w = max_workspace(B, N, T);
    char* base = static_cast<char*>(workspace);
    if (scan_taken_max(B, N, T)) {  // the schedule lccrf_auto_algo reports for the dense call of this shape
        hipStream_t st = static_cast<hipStream_t>(stream);
        int32_t* pin = reinterpret_cast<int32_t*>(base + w.pin);
        hipError_t e = lccrf::launch_scan_pins(
            LCCRF_F32, nullptr, lengths, B, N, T, scan_chunk_max(B, N, T), reinterpret_cast<double*>(base + w.Mx),
            reinterpret_cast<uint8_t*>(base + w.K), pin,
            {reinterpret_cast<double*>(base + w.Mx2), reinterpret_cast<uint8_t*>(base + w.K2),
             reinterpret_cast<int32_t*>(base + w.pin2)},
            best_score, st, emit, trans);
        if (e == hipSuccess)
            e = lccrf::launch_chunked_max(LCCRF_F32, nullptr, lengths, B, N, T, reinterpret_cast<uint8_t*>(base + w.bp),
                                          reinterpret_cast<double*>(base + w.mid), tags, scan_chunk_max(B, N, T), pin, st,
                                          emit, trans);
        return e == hipSuccess ? LCCRF_OK : LCCRF_ELAUNCH;
    }
    const hipError_t e = lccrf::launch_structured_max(emit, trans, lengths, B, N, T,
                                                      reinterpret_cast<uint8_t*>(base + w.bp),
                                                      reinterpret_cast<double*>(base + w.mid), best_score, tags,
                                                      static_cast<hipStream_t>(stream), lanes_pay_max(B, N, T),
                                                      g_lane_poll_limit.load(std::memory_order_relaxed));
    return e == hipSuccess ? LCCRF_OK : LCCRF_ELAUNCH;
}

const char* lccrf_strerror(int code) {
    switch (code) {
        case LCCRF_OK: return "ok";
        case LCCRF_EINVAL: return "invalid argument (B, N, T, dtype, op or algo)";
        case LCCRF_ENULL: return "a required pointer is NULL";
        case LCCRF_EWORKSPACE: return "workspace is NULL or too small";
        case LCCRF_EALIGN: return "a buffer is misaligned";
        case LCCRF_ELAUNCH: return "the HIP runtime refused a kernel launch";
        case LCCRF_ENOTIMPL: return "the requested schedule is not available for this shape";
        case LCCRF_ETOOBIG: return "the shape needs more scratch than the library's built-in buffer holds";
        default: return "unknown lccrf status";
    }
}

int lccrf_set_scan_chunk(int chunk) {
    if (chunk != 0 && (chunk < 4 || chunk > 4096)) return LCCRF_EINVAL;
    g_scan_chunk_user.store(chunk, std::memory_order_relaxed);
    return LCCRF_OK;
}

int lccrf_set_pair_poll_limit(int polls) {
    if (polls < -1 || polls > (1 << 24)) return LCCRF_EINVAL;
    g_pair_poll_limit.store(polls < 0 ? kDefaultPairPollLimit : polls, std::memory_order_relaxed);
    return LCCRF_OK;
}

int lccrf_set_lane_poll_limit(int polls) {
    if (polls < -1 || polls > (1 << 24)) return LCCRF_EINVAL;
    g_lane_poll_limit.store(polls < 0 ? kDefaultLanePollLimit : polls, std::memory_order_relaxed);
    return LCCRF_OK;
}

int lccrf_version(void) { return 201; }

}  // extern "C"
