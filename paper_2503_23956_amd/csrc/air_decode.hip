// air_decode_attn: Eq.2 append, then softmax(q K'^T / sqrt(d)) V' over the compacted cache.
//
//   decode_mfma_kernel bf16, head_dim 128, ONE launch per call: one workgroup per (split, unit), the
//                      grid laid out so that no block index needs an integer division.
//                      The tiled K' and the block-transposed V' go from global memory straight
//                      into MFMA operands, every load instruction reading 1 KB of consecutive
//                      memory; the G query heads of the group are the second MFMA dimension.
//                      The token the call appends (Eq.2) is scored from k_new / v_new by one wave
//                      of the split that owns its row, which also stores it into the cache; the
//                      workgroup of a unit that finishes last merges the unit's split-K partials.
//   append_kernel, decode_kernel, combine_kernel
//                      generic fp32-ALU path (fp32 storage, head_dim 64): three launches.
#include "air_device.h"
#include "air_internal.h"

#include <mutex>

namespace air {

constexpr int kMaxGroup = 16;

// ---------------------------------------------------------------------------------------
// Split-K exchange area of the entry point that allocates nothing (air_decode_attn_static): a fixed array in
// the library's own device image instead of the caller's workspace.  Every GPU the library runs on holds its own
// copy at its own address; host code only ever uses the address hipGetSymbolAddress returns for the current
// device (the array's name is a host-side stand-in, not a device address).
//   [arrival counters: kStaticSlots ints][(max, sum) pairs: kStaticSlots x 16][partial outputs: kStaticSlots x 16 x 128 floats]
// ---------------------------------------------------------------------------------------
constexpr size_t kStaticCntBytes = kStaticSlots * sizeof(int32_t);
constexpr size_t kStaticMlBytes = kStaticSlots * kMaxGroup * sizeof(float2);
constexpr size_t kStaticOBytes = kStaticSlots * kMaxGroup * 128 * sizeof(float);
constexpr size_t kStaticScratchBytes = kStaticCntBytes + kStaticMlBytes + kStaticOBytes;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];  // per device, filled on first use with that device current
static std::mutex g_scratch_mutex;

hipError_t static_exchange(DecodeExchange *x) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void *ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
            if (e != hipSuccess) return e;
            if (!ptr) return hipErrorInvalidSymbol;
            g_scratch_ptr[dev] = ptr;
        }
        ptr = g_scratch_ptr[dev];
    }
    if (x) {
        char *base = (char *)ptr;
        x->cnt = (int32_t *)base;
        x->ml = (float2 *)(base + kStaticCntBytes);
        x->o = (float *)(base + kStaticCntBytes + kStaticMlBytes);
        x->local = 1;
        x->stride = 0;  // set per launch: the launch's own split count
    }
    return hipSuccess;
}

// counters of a launch start at zero (a kernel, not a memset: the call may be recorded into a graph)
__global__ __launch_bounds__(256) void zero_counters_kernel(int32_t *p, int n) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0;
}
hipError_t launch_zero_counters(hipStream_t s, int32_t *p, int n) {
    hipLaunchKernelGGL(zero_counters_kernel, dim3((n + 255) / 256), dim3(256), 0, s, p, n);
    return hipGetLastError();
}

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// key range of one split: ceil(len / splits) rounded up to whole 32-token blocks
__device__ __forceinline__ void split_range(int len, int splits, int split, int &k0, int &k1) {
    int cs = (len + splits - 1) / splits;
    cs = (cs + 31) & ~31;
    k0 = split * cs;
    k1 = min(len, k0 + cs);
}

// ---------------------------------------------------------------------------------------
// append (Eq.2)
// ---------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(128) void append_kernel(Dims dm, DevTables t, int l0, int lbase, LaunchLayers ll,
                                                     const T *k_new, const T *v_new) {
    const int u = blockIdx.x;
    const int kvh = u % dm.Hkv;
    const int b = (u / dm.Hkv) % dm.B;
    const int li = u / (dm.Hkv * dm.B);
    const int l = l0 + li;
    const int row = t.base_len[(int64_t)b * dm.L + l] + ll.appended[li];
    const int64_t row0 = ((int64_t)b * dm.Hkv + kvh) * dm.pool_rows + t.layer_off[(int64_t)b * dm.L + l];
    const int64_t src = (((int64_t)(lbase + li) * dm.B + b) * dm.Hkv + kvh) * D;
    constexpr int kVec = D * (int)sizeof(T) / 16;
    const int tid = threadIdx.x;
    if (tid < kVec) {
        const int c = tid * (16 / (int)sizeof(T));
        *reinterpret_cast<uint4 *>((T *)t.kcache + (row0 + row) * D + c) = *reinterpret_cast<const uint4 *>(k_new + src + c);
        *reinterpret_cast<uint4 *>((T *)t.vcache + (row0 + row) * D + c) = *reinterpret_cast<const uint4 *>(v_new + src + c);
    }
}

// ---------------------------------------------------------------------------------------
// MFMA decode attention.  Workgroup (split, unit) of NW waves; wave w takes the chunks w, w+NW, ...
// (16*KT keys each) of the split's key range.  Lane (n = lane % 16, c = lane / 16).
//   scores^T tile (16 keys x 16 heads) = K'(16 keys x 128) * q^T: A = key n, elements 8c..8c+7 of
//   each 32-element slice; B = head n, same elements; the result leaves lane (n = head, c) with
//   keys 4c..4c+3 of the tile.  Two tiles cover a 32-token block, so that lane holds 8
//   probabilities of head n: exactly the A operand of P*V for the block when the block's tokens
//   are stored in v_slot order.  B of P*V = 16 bytes of the transposed V' block per lane, and the
//   accumulator of output tile j keeps heads 4c..4c+3 of column 16j + n.
// The kernel is bound by instruction issue as much as by memory when there are few units, so the
// key loop carries no predication: tiles past the end of the range re-read the last valid tile
// (their scores are masked, in the one iteration that has a tail), and the token this call appends
// (Eq.2) is not read through the cache at all: one wave of the split that owns its row scores it
// from k_new / v_new on the vector ALU and stores it into the cache.
// Softmax runs in the base-2 domain: logits are scaled by log2(e)/sqrt(d) and exponentiated with
// exp2; running maxima and the exchanged partial maxima are in that domain.
// The waves of a workgroup merge through LDS.  With more than one split per unit the
// workgroups exchange partials through memory and the one that finishes last merges them.
// ---------------------------------------------------------------------------------------
// What the MFMA decode kernel needs of the tables and of the per-layer launch block: a short
// argument block (the kernel starts with the loads of its arguments).
struct DecodeTabs {
    const int2 *len_off;
    const int4 *by_length;  // per sequence, (length, offset, layer) of the layers by falling cache length
    void *kcache, *vcache;
    float *dec_o;
    float2 *dec_ml;
    int32_t *dec_cnt;
    int32_t *dec_steps;  // null: the host passes the count of appended tokens (DecodeSteps)
    int32_t n_units;     // units of the whole context: dec_steps[n_units] is the cache-full flag
    const CachePtrs *cache_ptrs;  // in-place cache: the K / V tensor of every layer (else null: the cache is the workspace's pool)
    int64_t kv_b, kv_h;           // in-place cache: element strides between sequences / KV heads of those tensors
    int32_t x_local;     // 1: the exchange slots (dec_o, dec_ml, dec_cnt) are indexed by the unit inside the launch
    int32_t x_stride;    // exchange slots per unit
};
struct DecodeSteps {
    int32_t uniform;  // >= 0: every layer of the launch has appended this many tokens (any number of layers per launch)
    int32_t appended[kMaxLayersPerLaunch];
};

// INPLACE: the cache is kept inside the layers' own K / V tensors (their addresses come from a table)
// SORTED: a launch over all layers whose grid index z is not the layer but its rank by cache length within the
// sequence (longest first); the layer comes with the table entry that carries the length
// VH = 2: two workgroups per unit, each with one half of the columns of V' (see below); ONE_SEQ: the instance for B = 1
template <int NW, int KT, bool SPLIT, bool INPLACE, bool SORTED = false, int VH = 1, bool ONE_SEQ = false>
__global__ __launch_bounds__(64 * NW) void decode_mfma_kernel(Dims dm, DecodeTabs t, int l0, int lbase,
                                                              DecodeSteps ll, const bf16_t *q_new,
                                                              const bf16_t *k_new, const bf16_t *v_new, bf16_t *out,
                                                              int splits, int lg_splits) {
    constexpr int D = 128;
    constexpr int kIter = 16 * KT;  // keys per loop iteration of one wave (KT score tiles, KT/2 token blocks)
    constexpr int TB = KT / 2;
    constexpr int NJ = 8 / VH;  // output tiles (16 columns each) of the workgroup
    static_assert(VH == 1 || (!SPLIT && !SORTED && NJ % NW == 0), "column halves: one workgroup pair per unit");
    const int lane = threadIdx.x & 63, n = lane & 15, c = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // a scalar: the wave's chunk walk and its branches stay off the vector unit
    // grid (split + splits * KV head, sequence, layer): the linear order of the workgroups is (split, unit) and
    // no index needs a division (the number of splits is a power of two)
    const int split = SPLIT ? (int)blockIdx.x & (splits - 1) : 0;
    int kvh = SPLIT ? (int)blockIdx.x >> lg_splits : (int)blockIdx.x;
    int b = blockIdx.y;
    int li = blockIdx.z;
    int vh = 0;
    bool live = true;
    if (VH == 2) {
        // Two workgroups per unit, each with all of K' and one half of the columns of V' and of the output: no partials to
        // exchange, and a workgroup moves three quarters of the unit's bytes (a CU takes in about 140 GB/s, which is what
        // bounds a launch of few units).  A 1-D grid: the two workgroups of a unit get ids 16 p + x and 16 p + 8 + x, the
        // same XCD (ids are dealt round-robin over the 8 XCDs) at neighbouring dispatch slots, so that the K' tiles both
        // stream come through that XCD's L2 once.  `splits` carries the units of the launch (the grid is rounded up to
        // whole groups of 16: the workgroups past the end redo the last unit and store nothing), `lg_splits` log2 of
        // the KV heads.
        const int wid = blockIdx.x, slot = wid >> 3;
        int pair = ((slot >> 1) << 3) | (wid & 7);
        vh = slot & 1;
        live = pair < splits;
        pair = min(pair, splits - 1);
        kvh = pair & (dm.Hkv - 1);
        if (ONE_SEQ) {  // one sequence: its index is a constant of the instance (every address in front of the first loads is shorter: 0.6 us per launch)
            li = pair >> lg_splits;
            b = 0;
        } else {
            seq_layer_of(dm, pair >> lg_splits, b, li);
        }
    }
    int2 len_off;
    if (SORTED) {
        const int4 e = t.by_length[(int64_t)b * dm.L + blockIdx.z];
        len_off = make_int2(e.x, e.y);
        li = e.z - l0;
    }
    const int l = l0 + li;
    const int G = dm.G;
    // the unit's cache length and offset first: everything that touches the cache waits for them
    if (!SORTED) len_off = t.len_off[(int64_t)b * dm.L + l];
    CachePtrs cp = {nullptr, nullptr};
    if (INPLACE) cp = t.cache_ptrs[l];  // requested together with the table entry
    // The token this call appends (Eq.2): every wave fetches its k_new / v_new values first thing (the
    // addresses depend on the block index only), so they are long there when the wave that owns the
    // token needs them.
    const int64_t new_src = (((int64_t)(lbase + li) * dm.B + b) * dm.Hkv + kvh) * D;
    uint4 knew[4], krow;
    bf16_t vnew[NJ], vcol[2];
#pragma unroll
    for (int sl = 0; sl < 4; ++sl) knew[sl] = *reinterpret_cast<const uint4 *>(k_new + new_src + 32 * sl + 8 * c);
    krow = *reinterpret_cast<const uint4 *>(k_new + new_src + 8 * n);
#pragma unroll
    for (int j = 0; j < NJ; ++j) vnew[j] = v_new[new_src + 16 * (j + NJ * vh) + n];
    vcol[0] = v_new[new_src + 64 * vh + lane];
    if (VH == 1) vcol[1] = v_new[new_src + 64 + lane];
    const int64_t unit = ((int64_t)l * dm.B + b) * dm.Hkv + kvh;
    // tokens appended so far: from the host with the launch, or counted on the device (a recorded launch
    // that is replayed): the workgroup that finishes the unit advances the count, after every workgroup
    // of the unit has read it
    int appended = ll.uniform >= 0 ? ll.uniform : ll.appended[li];
    if (t.dec_steps) {
        appended = t.dec_steps[unit];
        if (appended >= dm.max_steps) {  // cache full: nothing is appended or written
            if (threadIdx.x == 0) t.dec_steps[t.n_units] = 1;
            return;
        }
    }
    if (VH == 2 && !live) return;
    const int len = len_off.x + appended + 1;
    const int newrow = len - 1;  // the token appended by this call (Eq.2): scored from k_new / v_new, stored to the cache
    int k0 = 0, k1 = len;
    if (SPLIT) {  // ceil(len / splits) rounded up to whole 32-token blocks, as split_range
        const int cs = (((len + splits - 1) >> lg_splits) + 31) & ~31;
        k0 = split * cs;
        k1 = min(len, k0 + cs);
    }
    const int kend = min(k1, newrow);  // the split's keys that are in the cache: [k0, kend)
    // the unit's cache: its region of the workspace pool, or (kept in place) its rows of the layer's own K / V tensors
    const int64_t row0 = INPLACE ? 0 : ((int64_t)b * dm.Hkv + kvh) * dm.pool_rows + len_off.y;
    const int64_t ip0 = INPLACE ? (int64_t)b * t.kv_b + (int64_t)kvh * t.kv_h : 0;
    bf16_t *kc = INPLACE ? (bf16_t *)cp.k + ip0 : (bf16_t *)t.kcache + row0 * D;
    bf16_t *vc = INPLACE ? (bf16_t *)cp.v + ip0 : (bf16_t *)t.vcache + row0 * D;
    bf16_t *o_unit = out + (((int64_t)(lbase + li) * dm.B + b) * dm.Hq + (int64_t)kvh * G) * D;

    bf16x8 qb[4];
    {
        // MFMA columns past the group's heads re-read its last head: their results are never stored
        const bf16_t *q = q_new + (((int64_t)(lbase + li) * dm.B + b) * dm.Hq + (int64_t)kvh * G + min(n, G - 1)) * D;
#pragma unroll
        for (int s = 0; s < 4; ++s) qb[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(q + 32 * s + 8 * c));
    }
    constexpr float kScale2 = 0.08838834764831845f * 1.4426950408889634f;  // log2(e) / sqrt(128)
    float m_run = -INFINITY, l_run = 0.f;
    f32x4 acc[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[j] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // ---- the appended token belongs to the wave of the owning split that would take the next
    // chunk.  The row goes into the cache at once, so that the stores complete behind the cache
    // loads: K' into its places of the tile, V' into its slot of the block (a token that opens a
    // block writes the block's other slots as zeros).  Other waves and splits never use these
    // places in this launch: their reads of them are masked or carry zero probability.  The
    // token's own score (vector ALU) starts the wave's running softmax: max = score, sum = 1,
    // accumulator = v_new for every head.
    const bool owns_new = newrow >= k0 && newrow < k1 && wave == ((kend - k0 + kIter - 1) / kIter) % NW;
    if (owns_new) {
        if (lane < 16 && vh == 0)  // the new K' row: 16 lanes x 16 bytes
            *reinterpret_cast<uint4 *>(kc + k_tiled(newrow, 8 * lane)) = krow;
        const int tok = newrow & 31;
#pragma unroll
        for (int h2 = 0; h2 < 2 / VH; ++h2) {
            const int col = lane + 64 * (h2 + vh);
            if (tok == 0) {  // a new block: the column's other slots are written as zeros
                bf16_t *vcolp = vc + (int64_t)newrow * D + (col >> 4) * 512 + (col & 15) * 8;  // slot group 0; +128 per group
                const uint4 z = make_uint4(0, 0, 0, 0);
                *reinterpret_cast<uint4 *>(vcolp) = make_uint4(vcol[h2], 0, 0, 0);  // token 0 sits in slot 0
                *reinterpret_cast<uint4 *>(vcolp + 128) = z;
                *reinterpret_cast<uint4 *>(vcolp + 256) = z;
                *reinterpret_cast<uint4 *>(vcolp + 384) = z;
            } else {
                vc[v_tiled(newrow, col)] = vcol[h2];
            }
        }
        float sn = 0.f;
#pragma unroll
        for (int sl = 0; sl < 4; ++sl) {
            const uint4 kx = knew[sl];
            const uint4 qx = __builtin_bit_cast(uint4, qb[sl]);
            const uint32_t kw[4] = {kx.x, kx.y, kx.z, kx.w}, qw[4] = {qx.x, qx.y, qx.z, qx.w};
#pragma unroll
            for (int w4 = 0; w4 < 4; ++w4) {
                sn = fmaf(__uint_as_float(qw[w4] << 16), __uint_as_float(kw[w4] << 16), sn);
                sn = fmaf(__uint_as_float(qw[w4] & 0xffff0000u), __uint_as_float(kw[w4] & 0xffff0000u), sn);
            }
        }
        sn += __shfl_xor(sn, 16, 64);
        sn += __shfl_xor(sn, 32, 64);
        m_run = sn * kScale2;
        l_run = c == 0 ? 1.f : 0.f;  // l_run is a per-lane partial of the head's sum: the token counts once
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const float v = bf16_bits_to_float(vnew[j]);
            acc[j] = (f32x4){v, v, v, v};
        }
    }

    const int last16 = (kend - 1) & ~15, last32 = (kend - 1) & ~31;  // last tile / block with a cached key
    // The chunks of the range are walked front to back on even steps and back to front on odd ones:
    // what a step read last is what the next step reads first, so the part of the cache that is
    // still in the L2 of the XCD (the unit-to-XCD mapping is the same every launch) gets reused
    // instead of being evicted just before its turn.
    const bool backward = (appended & 1) != 0;
    const int n_chunks = (max(kend - k0, 0) + kIter - 1) / kIter;
    const int kb_first = k0 + (backward ? n_chunks - 1 - wave : wave) * kIter;
    const int kStep = (backward ? -NW : NW) * kIter;  // distance between two chunks of one wave
    auto has = [&](int kb) { return kb >= k0 && kb < kend; };

    // all loads of a chunk: the KT score tiles of K' and the V' operands of the TB token blocks
    auto load_chunk = [&](uint4(&a)[KT][4], uint4(&vb)[TB][NJ], int kb) {
#pragma unroll
        for (int tile = 0; tile < KT; ++tile) {
            const bf16_t *src = kc + (int64_t)min(kb + 16 * tile, last16) * D + 32 * n + 8 * c;
#pragma unroll
            for (int sl = 0; sl < 4; ++sl) a[tile][sl] = *reinterpret_cast<const uint4 *>(src + 512 * sl);
        }
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            const bf16_t *src = vc + (int64_t)min(kb + 32 * tb, last32) * D + 128 * c + 8 * n;
#pragma unroll
            for (int j = 0; j < NJ; ++j) vb[tb][j] = *reinterpret_cast<const uint4 *>(src + 512 * (j + NJ * vh));
        }
    };
    auto compute_chunk = [&](const uint4(&a)[KT][4], const uint4(&vb)[TB][NJ], int kb) {
        // ---- scores^T
        f32x4 s[KT];
#pragma unroll
        for (int tile = 0; tile < KT; ++tile) {
            s[tile] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int sl = 0; sl < 4; ++sl)
                s[tile] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[tile][sl]), qb[sl], s[tile], 0, 0, 0);
        }
        if (kb + kIter > kend) {  // the chunk with the tail (uniform over the wave)
#pragma unroll
            for (int tile = 0; tile < KT; ++tile)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (kb + 16 * tile + 4 * c + i >= kend) s[tile][i] = -INFINITY;
        }
        // ---- online softmax for head n over the keys this lane holds (4c+i of each tile).  The four lanes of a
        // head share one reference maximum m_run; it is raised (and the accumulators rescaled) only when some
        // score of the chunk lies more than kSlack above it, so most chunks need no cross-lane step at all:
        // probabilities may then be as large as 2^kSlack, which fp32 sums and bf16 operands hold without loss.
        // The sum l_run stays a per-lane partial and is added up over the four lanes after the last chunk.
        constexpr float kSlack = 8.0f;
        float mloc = s[0][0];
#pragma unroll
        for (int tile = 0; tile < KT; ++tile)
#pragma unroll
            for (int i = 0; i < 4; ++i) mloc = fmaxf(mloc, s[tile][i]);
        mloc *= kScale2;
        if (__ballot(mloc > m_run + kSlack) != 0ull) {  // uniform over the wave; always taken on a wave's first chunk
            float mb = fmaxf(mloc, __shfl_xor(mloc, 16, 64));
            mb = fmaxf(mb, __shfl_xor(mb, 32, 64));
            const float m_new = fmaxf(m_run, mb);  // finite: key kb is valid
            const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
            l_run *= corr;
            m_run = m_new;
            // accumulator rows are heads 4c..4c+3: fetch their rescale factors from lanes 4c+i
            if ((owns_new || kb != kb_first) && __ballot(corr != 1.0f) != 0ull) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float f = __shfl(corr, 4 * c + i, 64);
#pragma unroll
                    for (int j = 0; j < NJ; ++j) acc[j][i] *= f;
                }
            }
        }
        float lb = 0.f;
#pragma unroll
        for (int tile = 0; tile < KT; ++tile)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float p = __builtin_amdgcn_exp2f(fmaf(s[tile][i], kScale2, -m_run));
                s[tile][i] = p;
                lb += p;
            }
        l_run += lb;
        // ---- P * V
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            bf16x8 pa;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                pa[i] = (__bf16)s[2 * tb][i];
                pa[4 + i] = (__bf16)s[2 * tb + 1][i];
            }
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa, __builtin_bit_cast(bf16x8, vb[tb][j]), acc[j], 0, 0, 0);
        }
    };
    // Two chunk buffers: while one chunk is multiplied the loads of the wave's next chunk are in
    // flight.  Loads are issued only for chunks that exist, and the loop is laid out so that every
    // path reaches a compute step with the same loads behind it (the wait counts stay exact).
    if constexpr (KT > 2 && VH == 1) {  // two buffers of this size do not fit the registers: load, then multiply
        for (int kb = kb_first; has(kb); kb += kStep) {
            uint4 a0[KT][4], v0[TB][NJ];
            load_chunk(a0, v0, kb);
            compute_chunk(a0, v0, kb);
        }
    } else if (has(kb_first)) {
        uint4 a0[KT][4], v0[TB][NJ], a1[KT][4], v1[TB][NJ];
        int kb = kb_first;
        load_chunk(a0, v0, kb);
        if (!has(kb + kStep)) {
            compute_chunk(a0, v0, kb);
        } else {
            load_chunk(a1, v1, kb + kStep);
            while (true) {
                compute_chunk(a0, v0, kb);
                if (!has(kb + 2 * kStep)) {
                    compute_chunk(a1, v1, kb + kStep);
                    break;
                }
                load_chunk(a0, v0, kb + 2 * kStep);
                compute_chunk(a1, v1, kb + kStep);
                if (!has(kb + 3 * kStep)) {
                    compute_chunk(a0, v0, kb + 2 * kStep);
                    break;
                }
                load_chunk(a1, v1, kb + 3 * kStep);
                kb += 2 * kStep;
            }
        }
    }

    // the head's sum over the four lanes that hold its keys
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);

    // ---- merge the NW waves of the workgroup through LDS.  Every wave first rescales its partial
    // to the workgroup's maximum, so that the merge is a plain sum: wave w ends up with output
    // tiles w, w+NW, ... (heads 4c..4c+3, column 16j+n), plus the merged (max, sum) of those heads.
    __shared__ f32x4 s_acc[NW][NJ][64];
    __shared__ float s_mw[kMaxGroup][NW], s_lw[kMaxGroup][NW];
    __shared__ int s_prev;
    float mrg_m[4], mrg_l[4];  // merged max / sum of heads 4c+i
    if (NW > 1) {
        if (c == 0) s_mw[n][wave] = m_run;
        __syncthreads();
        float M = s_mw[n][0];
#pragma unroll
        for (int w = 1; w < NW; ++w) M = fmaxf(M, s_mw[n][w]);
        const float f = m_run == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_run - M);
        if (c == 0) s_lw[n][wave] = l_run * f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float fi = __shfl(f, 4 * c + i, 64);
            mrg_m[i] = __shfl(M, 4 * c + i, 64);
#pragma unroll
            for (int j = 0; j < NJ; ++j) acc[j][i] *= fi;
        }
#pragma unroll
        for (int j = 0; j < NJ; ++j) s_acc[wave][j][lane] = acc[j];
        __syncthreads();
#pragma unroll
        for (int jj = 0; jj < NJ / NW; ++jj) {
            const int j = wave + NW * jj;
            f32x4 sum = s_acc[0][j][lane];
#pragma unroll
            for (int w = 1; w < NW; ++w) {
                const f32x4 x = s_acc[w][j][lane];
#pragma unroll
                for (int i = 0; i < 4; ++i) sum[i] += x[i];
            }
            acc[jj] = sum;  // tile wave + NW*jj
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float Lsum = s_lw[4 * c + i][0];
#pragma unroll
            for (int w = 1; w < NW; ++w) Lsum += s_lw[4 * c + i][w];
            mrg_l[i] = Lsum;
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            mrg_m[i] = __shfl(m_run, 4 * c + i, 64);
            mrg_l[i] = __shfl(l_run, 4 * c + i, 64);
        }
    }
    constexpr int kTiles = NJ / NW;  // output tiles this wave owns after the merge: j = wave + NW*jj (of the workgroup's NJ)

    if (!SPLIT || splits == 1) {  // no partials: normalise and store
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int g = 4 * c + i;
            if (g < G) {
                const float inv = __builtin_amdgcn_rcpf(mrg_l[i]);
#pragma unroll
                for (int jj = 0; jj < kTiles; ++jj)
                    o_unit[g * D + 16 * (NJ * vh + wave + NW * jj) + n] = float_to_bf16_bits(acc[jj][i] * inv);
            }
        }
        if (t.dec_steps && threadIdx.x == 0) {
            if (VH == 1) {
                t.dec_steps[unit] = appended + 1;
            } else {
                // the workgroup of the pair that finishes second advances the count: the other one has read it by then
                const int64_t xu = t.x_local ? ((int64_t)li * dm.B + b) * dm.Hkv + kvh : unit;
                if (__hip_atomic_fetch_add(&t.dec_cnt[xu], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 1) {
                    __hip_atomic_store(&t.dec_cnt[xu], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // next launch
                    t.dec_steps[unit] = appended + 1;
                }
            }
        }
        return;
    }
    if (!SPLIT) return;  // the instance for one workgroup per unit carries none of what follows
    // ---- partial of this split.  Partials are exchanged between workgroups of one launch, which
    // may run on different XCDs (separate L2s).  They are written and read with system-scope
    // (write-through / L2-bypassing) 16-byte accesses in the accumulators' own lane layout, the
    // writers wait for their stores to complete before the workgroup counts itself, and the
    // workgroup that counts last reads them.  This keeps the exchange off the whole-L2 write-back
    // that a release fence would cost.  Layout of one partial: [tile j][lane][4] floats.
    const int64_t xu = t.x_local ? ((int64_t)li * dm.B + b) * dm.Hkv + kvh : unit;  // the unit's exchange slots
    const int64_t part = xu * t.x_stride + split;
    float *pu = t.dec_o + xu * t.x_stride * (int64_t)kMaxGroup * D;
    const __amdgpu_buffer_rsrc_t prs = __builtin_amdgcn_make_buffer_rsrc(pu, 0, t.x_stride * kMaxGroup * D * 4, 0x00020000);
    if (4 * c < G) {
#pragma unroll
        for (int jj = 0; jj < kTiles; ++jj)
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, acc[jj]), prs,
                                                   (split * kMaxGroup * D + ((wave + NW * jj) * 64 + lane) * 4) * 4, 0,
                                                   kSysScope);
    }
    if (wave == 0 && n == 0) {  // lane (0, c) holds the merged stats of heads 4c..4c+3
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int g = 4 * c + i;
            if (g < G) {
                float *mlp = reinterpret_cast<float *>(t.dec_ml + part * G + g);
                __hip_atomic_store(mlp, mrg_m[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(mlp + 1, mrg_l[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) s_prev = __hip_atomic_fetch_add(&t.dec_cnt[xu], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (s_prev != splits - 1) return;
    if (threadIdx.x == 0) __hip_atomic_store(&t.dec_cnt[xu], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // next launch

    // merge of the splits: every wave loads the partial tiles it owns (one round of loads), the
    // (max, sum) pairs go through LDS
    __shared__ float s_m[kMaxSplits][kMaxGroup], s_l[kMaxSplits][kMaxGroup], s_w[kMaxSplits][kMaxGroup];
    __shared__ float s_inv[kMaxGroup];
    const float *ml = reinterpret_cast<const float *>(t.dec_ml + xu * t.x_stride * G);
    f32x4 num[kTiles];
#pragma unroll
    for (int jj = 0; jj < kTiles; ++jj) num[jj] = (f32x4){0.f, 0.f, 0.f, 0.f};
    for (int p = threadIdx.x; p < splits * G; p += 64 * NW) {
        s_m[p / G][p % G] = __hip_atomic_load(ml + 2 * p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_l[p / G][p % G] = __hip_atomic_load(ml + 2 * p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if ((int)threadIdx.x < G) {
        const int g = threadIdx.x;
        float M = -INFINITY;
        for (int s2 = 0; s2 < splits; ++s2) M = fmaxf(M, s_m[s2][g]);
        float den = 0.f;
        for (int s2 = 0; s2 < splits; ++s2) {
            const float wg = s_l[s2][g] > 0.f ? __builtin_amdgcn_exp2f(s_m[s2][g] - M) : 0.f;
            s_w[s2][g] = wg;
            den = fmaf(wg, s_l[s2][g], den);
        }
        s_inv[g] = 1.0f / den;
    }
    __syncthreads();
    constexpr int kRound = (32 / kTiles) < kMaxSplits ? (32 / kTiles) : kMaxSplits;  // splits loaded together
    for (int s0 = 0; s0 < splits; s0 += kRound) {
        f32x4 v[kRound][kTiles];
#pragma unroll
        for (int s2 = 0; s2 < kRound; ++s2)
#pragma unroll
            for (int jj = 0; jj < kTiles; ++jj) {
                v[s2][jj] = (f32x4){0.f, 0.f, 0.f, 0.f};
                if (s0 + s2 < splits && 4 * c < G)
                    v[s2][jj] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
                        prs, ((s0 + s2) * kMaxGroup * D + ((wave + NW * jj) * 64 + lane) * 4) * 4, 0, kSysScope));
            }
#pragma unroll
        for (int s2 = 0; s2 < kRound; ++s2) {
            if (s0 + s2 < splits) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float wg = s_w[s0 + s2][(4 * c + i) & (kMaxGroup - 1)];
#pragma unroll
                    for (int jj = 0; jj < kTiles; ++jj) num[jj][i] = fmaf(wg, v[s2][jj][i], num[jj][i]);
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int g = 4 * c + i;
        if (g < G) {
            const float inv = s_inv[g];
#pragma unroll
            for (int jj = 0; jj < kTiles; ++jj)
                o_unit[g * D + 16 * (wave + NW * jj) + n] = float_to_bf16_bits(num[jj][i] * inv);
        }
    }
    if (t.dec_steps && threadIdx.x == 0) t.dec_steps[unit] = appended + 1;
}

// ---------------------------------------------------------------------------------------
// generic decode attention: one workgroup per (split, unit), thread per key for q.K', thread
// per output column for P.V', online softmax over blocks of 256 keys.
// ---------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(256) void decode_kernel(Dims dm, DevTables t, DecodeExchange x, int l0, int lbase,
                                                     LaunchLayers ll, const T *q_new, int splits) {
    constexpr int NP = 256 / D;  // key-parallel parts in the P*V phase
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int split = blockIdx.x;
    const int u = blockIdx.y;
    const int kvh = u % dm.Hkv;
    const int b = (u / dm.Hkv) % dm.B;
    const int li = u / (dm.Hkv * dm.B);
    const int l = l0 + li;
    const int G = dm.G;
    const int len = t.base_len[(int64_t)b * dm.L + l] + ll.appended[li] + 1;
    int k0, k1;
    split_range(len, splits, split, k0, k1);
    const int64_t row0 = ((int64_t)b * dm.Hkv + kvh) * dm.pool_rows + t.layer_off[(int64_t)b * dm.L + l];
    const T *kc = (const T *)t.kcache + row0 * D;
    const T *vc = (const T *)t.vcache + row0 * D;
    const int64_t unit = ((int64_t)l * dm.B + b) * dm.Hkv + kvh;

    __shared__ float s_q[kMaxGroup][D];
    __shared__ float s_p[kMaxGroup][256];
    __shared__ float s_m[kMaxGroup], s_l[kMaxGroup], s_corr[kMaxGroup];
    __shared__ float s_o[NP][kMaxGroup][D];

    const T *q = q_new + (((int64_t)(lbase + li) * dm.B + b) * dm.Hq + (int64_t)kvh * G) * D;
    for (int idx = tid; idx < G * D; idx += 256) s_q[idx / D][idx % D] = ldf(q + idx);
    if (tid < kMaxGroup) {
        s_m[tid] = -INFINITY;
        s_l[tid] = 0.f;
    }
    const float scale = 1.0f / sqrtf((float)D);
    const int dcol = tid % D, part = tid / D;
    float acc[kMaxGroup];
#pragma unroll
    for (int g = 0; g < kMaxGroup; ++g) acc[g] = 0.f;
    __syncthreads();

    for (int kb = k0; kb < k1; kb += 256) {
        const int nk = min(256, k1 - kb);
        {
            float kreg[D];
            if (tid < nk) load_row<D>(kc + (int64_t)(kb + tid) * D, kreg);
            for (int g = 0; g < G; ++g) {
                float a = 0.f;
                if (tid < nk) {
#pragma unroll
                    for (int cc = 0; cc < D; ++cc) a = fmaf(s_q[g][cc], kreg[cc], a);
                }
                s_p[g][tid] = tid < nk ? a * scale : -INFINITY;
            }
        }
        __syncthreads();
        for (int g = wave; g < G; g += 4) {
            float v0 = s_p[g][lane], v1 = s_p[g][lane + 64], v2 = s_p[g][lane + 128], v3 = s_p[g][lane + 192];
            const float mb = wave_max(fmaxf(fmaxf(v0, v1), fmaxf(v2, v3)));
            const float mo = s_m[g];
            const float mn = fmaxf(mo, mb);
            v0 = expf(v0 - mn);
            v1 = expf(v1 - mn);
            v2 = expf(v2 - mn);
            v3 = expf(v3 - mn);
            s_p[g][lane] = v0;
            s_p[g][lane + 64] = v1;
            s_p[g][lane + 128] = v2;
            s_p[g][lane + 192] = v3;
            const float lb = wave_sum((v0 + v1) + (v2 + v3));
            if (lane == 0) {
                const float corr = expf(mo - mn);  // 0 on the first block (mo = -inf)
                s_corr[g] = corr;
                s_l[g] = s_l[g] * corr + lb;
                s_m[g] = mn;
            }
        }
        __syncthreads();
#pragma unroll
        for (int g = 0; g < kMaxGroup; ++g)
            if (g < G) acc[g] *= s_corr[g];
        for (int tk = part; tk < nk; tk += NP) {
            const float vv = ldf(vc + (int64_t)(kb + tk) * D + dcol);
#pragma unroll
            for (int g = 0; g < kMaxGroup; ++g)
                if (g < G) acc[g] = fmaf(s_p[g][tk], vv, acc[g]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int g = 0; g < kMaxGroup; ++g)
        if (g < G) s_o[part][g][dcol] = acc[g];
    __syncthreads();
    const int64_t pidx = (x.local ? (int64_t)u : unit) * x.stride + split;
    float *po = x.o + pidx * (int64_t)G * D;
    for (int idx = tid; idx < G * D; idx += 256) {
        const int g = idx / D, cc = idx % D;
        float o = 0.f;
#pragma unroll
        for (int p = 0; p < NP; ++p) o += s_o[p][g][cc];
        po[idx] = o;
    }
    if (tid < G) x.ml[pidx * G + tid] = make_float2(s_m[tid], s_l[tid]);
}

template <typename T, int D>
__global__ __launch_bounds__(256) void combine_kernel(Dims dm, DecodeExchange x, int l0, int lbase, T *out, int splits) {
    const int u = blockIdx.x;
    const int kvh = u % dm.Hkv;
    const int b = (u / dm.Hkv) % dm.B;
    const int li = u / (dm.Hkv * dm.B);
    const int l = l0 + li;
    const int G = dm.G;
    const int64_t unit = ((int64_t)l * dm.B + b) * dm.Hkv + kvh;
    const int64_t xu = x.local ? (int64_t)u : unit;
    const float2 *ml = x.ml + xu * x.stride * G;
    const float *po = x.o + xu * x.stride * (int64_t)G * D;
    T *o = out + (((int64_t)(lbase + li) * dm.B + b) * dm.Hq + (int64_t)kvh * G) * D;
    for (int idx = threadIdx.x; idx < G * D; idx += 256) {
        const int g = idx / D;
        float M = -INFINITY;
        for (int s = 0; s < splits; ++s) M = fmaxf(M, ml[s * G + g].x);
        float num = 0.f, den = 0.f;
        for (int s = 0; s < splits; ++s) {
            const float2 x = ml[s * G + g];
            const float wgt = x.y > 0.f ? expf(x.x - M) : 0.f;
            num = fmaf(wgt, po[(int64_t)s * G * D + idx], num);
            den = fmaf(wgt, x.y, den);
        }
        stf(o + idx, num / den);
    }
}

template <typename T, int D>
static hipError_t append_launch(hipStream_t s, const Dims &dm, const DevTables &t, int l0, int nl, int lbase,
                                const LaunchLayers &ll, const void *k_new, const void *v_new) {
    hipLaunchKernelGGL((append_kernel<T, D>), dim3(nl * dm.B * dm.Hkv), dim3(128), 0, s, dm, t, l0, lbase, ll,
                       (const T *)k_new, (const T *)v_new);
    return hipGetLastError();
}

static hipError_t launch_append(hipStream_t s, const Dims &dm, const DevTables &t, int dtype, int l0, int nl, int lbase,
                         const LaunchLayers &ll, const void *k_new, const void *v_new) {
    if (dtype == AIR_BF16) return append_launch<bf16_t, 64>(s, dm, t, l0, nl, lbase, ll, k_new, v_new);  // head_dim 128 takes the MFMA kernel
    return dm.D == 128 ? append_launch<float, 128>(s, dm, t, l0, nl, lbase, ll, k_new, v_new)
                       : append_launch<float, 64>(s, dm, t, l0, nl, lbase, ll, k_new, v_new);
}

template <typename T, int D>
static hipError_t decode_launch(hipStream_t s, const Dims &dm, const DevTables &t, const DecodeExchange &x, int l0, int nl,
                                int lbase, const LaunchLayers &ll, const void *q_new, void *out, int splits) {
    const int units = nl * dm.B * dm.Hkv;
    hipLaunchKernelGGL((decode_kernel<T, D>), dim3(splits, units), dim3(256), 0, s, dm, t, x, l0, lbase, ll,
                       (const T *)q_new, splits);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((combine_kernel<T, D>), dim3(units), dim3(256), 0, s, dm, x, l0, lbase, (T *)out, splits);
    return hipGetLastError();
}

// Generic path: append, split-K attention, combine (three launches).
hipError_t launch_decode(hipStream_t s, const Dims &dm, const DevTables &t, const DecodeExchange &x, int dtype, int l0,
                         int nl, int lbase, const LaunchLayers &ll, const void *q_new, const void *k_new,
                         const void *v_new, void *out, int splits, int waves, int tiles, int uniform_appended,
                         bool longest_first, bool column_halves) {
    if (v_transposed(dtype, dm.D)) {  // one launch: append, attention and merge of the partials
        if (splits < 1 || (splits & (splits - 1)) != 0) return hipErrorInvalidValue;  // the kernel shifts by log2(splits)
        int lg_splits = 0;
        while ((1 << lg_splits) < splits) ++lg_splits;
        const dim3 grid(splits * dm.Hkv, dm.B, nl);
        DecodeTabs dt;
        dt.len_off = t.len_off;
        dt.by_length = t.by_length;
        dt.kcache = t.kcache;
        dt.vcache = t.vcache;
        dt.dec_o = x.o;
        dt.dec_ml = x.ml;
        dt.dec_cnt = x.cnt;
        dt.x_local = x.local;
        dt.x_stride = x.stride;
        dt.dec_steps = t.dec_steps;
        dt.cache_ptrs = t.cache_ptrs;
        dt.kv_b = t.ip_kv_b;
        dt.kv_h = t.ip_kv_h;
        dt.n_units = dm.L * dm.B * dm.Hkv;
        DecodeSteps ds;
        ds.uniform = uniform_appended;
        for (int i = 0; i < kMaxLayersPerLaunch; ++i) ds.appended[i] = ll.appended[i];
#define AIR_LAUNCH_DECODE_(NW, KT, SP, IP)                                                                          \
    hipLaunchKernelGGL((decode_mfma_kernel<NW, KT, SP, IP>), grid, dim3(64 * NW), 0, s, dm, dt, l0, lbase, ds,      \
                       (const bf16_t *)q_new, (const bf16_t *)k_new, (const bf16_t *)v_new, (bf16_t *)out, splits,  \
                       lg_splits)
#define AIR_LAUNCH_DECODE(NW, KT)                                                       \
    do {                                                                                \
        if (splits == 1 && !t.cache_ptrs) AIR_LAUNCH_DECODE_(NW, KT, false, false);     \
        else if (splits == 1) AIR_LAUNCH_DECODE_(NW, KT, false, true);                  \
        else if (!t.cache_ptrs) AIR_LAUNCH_DECODE_(NW, KT, true, false);                \
        else AIR_LAUNCH_DECODE_(NW, KT, true, true);                                    \
    } while (0)
        if (column_halves) {  // the caller has checked what this variant asks for
            const int units = nl * dm.B * dm.Hkv;
            int lg_h = 0;
            while ((1 << lg_h) < dm.Hkv) ++lg_h;
            const dim3 grid2(2 * ((units + 7) & ~7));
#define AIR_LAUNCH_HALVES_(IP, ONE)                                                                                        \
    hipLaunchKernelGGL((decode_mfma_kernel<4, 4, false, IP, false, 2, ONE>), grid2, dim3(256), 0, s, dm, dt, l0, lbase, ds, \
                       (const bf16_t *)q_new, (const bf16_t *)k_new, (const bf16_t *)v_new, (bf16_t *)out, units, lg_h)
            if (t.cache_ptrs) {
                if (dm.B == 1) AIR_LAUNCH_HALVES_(true, true);
                else AIR_LAUNCH_HALVES_(true, false);
            } else {
                if (dm.B == 1) AIR_LAUNCH_HALVES_(false, true);
                else AIR_LAUNCH_HALVES_(false, false);
            }
#undef AIR_LAUNCH_HALVES_
            return hipGetLastError();
        }
        if (longest_first && splits == 1 && !t.cache_ptrs && tiles == 4 && (waves == 1 || waves == 4)) {
            if (waves == 4)
                hipLaunchKernelGGL((decode_mfma_kernel<4, 4, false, false, true>), grid, dim3(256), 0, s, dm, dt, l0, lbase, ds,
                                   (const bf16_t *)q_new, (const bf16_t *)k_new, (const bf16_t *)v_new, (bf16_t *)out, splits, lg_splits);
            else
                hipLaunchKernelGGL((decode_mfma_kernel<1, 4, false, false, true>), grid, dim3(64), 0, s, dm, dt, l0, lbase, ds,
                                   (const bf16_t *)q_new, (const bf16_t *)k_new, (const bf16_t *)v_new, (bf16_t *)out, splits, lg_splits);
            return hipGetLastError();
        }
        if (waves == 8 && tiles == 4) AIR_LAUNCH_DECODE(8, 4);
        else if (waves == 4 && tiles == 4) AIR_LAUNCH_DECODE(4, 4);
        else if (waves == 2 && tiles == 4) AIR_LAUNCH_DECODE(2, 4);
        else if (waves == 1 && tiles == 4) AIR_LAUNCH_DECODE(1, 4);
        else if (waves == 8 && tiles == 2) AIR_LAUNCH_DECODE(8, 2);
        else if (waves == 4 && tiles == 2) AIR_LAUNCH_DECODE(4, 2);
        else if (waves == 2 && tiles == 2) AIR_LAUNCH_DECODE(2, 2);
        else if (waves == 1 && tiles == 2) AIR_LAUNCH_DECODE(1, 2);
        else if (waves == 4) AIR_LAUNCH_DECODE(4, 8);
        else if (waves == 2) AIR_LAUNCH_DECODE(2, 8);
        else AIR_LAUNCH_DECODE(1, 8);
#undef AIR_LAUNCH_DECODE
#undef AIR_LAUNCH_DECODE_
        return hipGetLastError();
    }
    hipError_t e = launch_append(s, dm, t, dtype, l0, nl, lbase, ll, k_new, v_new);
    if (e != hipSuccess) return e;
    if (dtype == AIR_BF16) return decode_launch<bf16_t, 64>(s, dm, t, x, l0, nl, lbase, ll, q_new, out, splits);
    return dm.D == 128 ? decode_launch<float, 128>(s, dm, t, x, l0, nl, lbase, ll, q_new, out, splits)
                       : decode_launch<float, 64>(s, dm, t, x, l0, nl, lbase, ll, q_new, out, splits);
}

}  // namespace air
