// MLP gradients at two iterates on the same minibatch (step a1; gradient of the sum of the
// per-sample softmax cross-entropy losses, paper Sec. II-A), with MFMA GEMMs.
//
// Model: a_0 = x; a_l = ReLU(W_l a_{l-1} + b_l) for l < L; logits = W_L a_{L-1} + b_L.
// For every group g the forward and backward passes run twice: at theta^k (shared by all
// groups) and at theta_stale_g = ring slot (k - tau_g).  The weight gradients of the two
// iterates are formed in the same workgroup, so that their difference (for stat_g) is taken
// in fp32 registers and only the fresh gradient is written.
//
// Every GEMM is brought to the form C[M][N] = sum_k P[M][k] Q[N][k] with both operands
// contiguous along k: activations and back-propagated signals are stored row-major AND
// transposed by the kernel that produces them, and the weights have a padded compute copy and a
// transposed copy per ring slot.  T is float (v_mfma_f32_32x32x2_f32) or bf16
// (v_mfma_f32_32x32x16_bf16); accumulation is fp32 in both cases.
#include <hip/hip_bf16.h>

#include "gcada_internal.h"

namespace gcada {

namespace {

constexpr int kWave = 64;
using bf16_t = __bf16;
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// float -> T -> float with round to nearest even (identity for float).  bf16: the conversion
// instruction of the hardware (v_cvt_pk_bf16_f32), not bit arithmetic.
template <typename T> __device__ __forceinline__ float round_to(float v);
template <> __device__ __forceinline__ float round_to<float>(float v) { return v; }
template <> __device__ __forceinline__ float round_to<bf16_t>(float v) { return (float)(bf16_t)v; }
template <typename T> __device__ __forceinline__ T to_T(float v);
template <> __device__ __forceinline__ float to_T<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t to_T<bf16_t>(float v) { return (bf16_t)v; }
// two floats -> one word of two bf16 (lo in the low half): one conversion instruction
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi)
{
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const f32x2 v = {lo, hi};
    const bf16x2 r = __builtin_convertvector(v, bf16x2);
    unsigned u;
    __builtin_memcpy(&u, &r, 4);
    return u;
}
template <typename T> __device__ __forceinline__ float to_f(T v);
template <> __device__ __forceinline__ float to_f<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f<bf16_t>(bf16_t v)
{
    unsigned short s;
    __builtin_memcpy(&s, &v, 2);
    return __uint_as_float((unsigned)s << 16);
}

__host__ __device__ inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

// ---------------------------------------------------------------------------------------
// Layout of one context's MLP work space (all leading dimensions are multiples of 64 elements
// and every pad element stays zero, so GEMM k-loops may run over the padding).
struct Layout {
    int L;                       // layers (widths - 1)
    int n[GCADA_MAX_WIDTHS];     // widths n_0..n_L
    int ld[GCADA_MAX_WIDTHS];    // round_up(n_l, 64)
    int ldmu;                    // round_up(mu, 64)
    int64_t woff[GCADA_MAX_WIDTHS];   // offset of W_l in theta (l = 1..L)
    int64_t boff[GCADA_MAX_WIDTHS];   // offset of b_l in theta
};

// ---------------------------------------------------------------------------------------
// GEMM  C[M][N] = sum_k P[M][k] Q[N][k],  BM x BN tile, WM x WN waves, each wave
// (BM/WM) x (BN/WN) as TM x TN blocks of 32 x 32.  A row of a tile in LDS is KROW bytes of k plus
// 16 bytes of padding.  Two LDS stages; PF = k-tiles in flight in registers ahead of the one
// being multiplied (1 or 2).
template <int BM_, int BN_, int KROW_, int WM_ = 2, int WN_ = 2, int PF_ = 1, int WPE_ = 1>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, KROW = KROW_, WM = WM_, WN = WN_, PF = PF_;
    static constexpr int WPE = WPE_;                         // waves per SIMD the kernel must leave room for
    static constexpr int NW = WM * WN, NT = NW * 64;          // waves, threads
    static constexpr int PITCH = KROW + 16;
    static constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    static constexpr int CPR = KROW / 16;                    // 16-byte chunks per row
    static constexpr int PCH = BM * CPR / NT, QCH = BN * CPR / NT;     // chunks per thread
    static constexpr int KS = KROW / 32;                     // 32-byte k-steps per tile
    static constexpr int STAGE = (BM + BN) * PITCH;
    static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0 && (BM * CPR) % NT == 0 && (BN * CPR) % NT == 0, "tile");
    static_assert(PF == 1 || PF == 2, "prefetch distance");
};
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int kHeadClasses = 128;             // the output layer's classes fit one tile

enum { EPI_FWD = 0, EPI_DA = 1, EPI_DW = 2, EPI_HEAD = 3 };

constexpr int cmax(int x, int y) { return x > y ? x : y; }
// dynamic LDS of a kernel: the two k-loop stages, or what its epilogue stages there
template <typename T, int EPI, typename TL>
constexpr int gemm_lds_bytes()
{
    const int loop = 2 * TL::STAGE;
    if (EPI == EPI_DW) return cmax(loop, 8 * TL::NW);
    if (EPI == EPI_HEAD) return cmax(loop, TL::BM * (TL::BN + 4) * 4 + 8 * TL::NW);
    constexpr int V = 16 / (int)sizeof(T);
    return cmax(loop, cmax(TL::BM * (TL::BN + V), TL::BN * (TL::BM + V)) * (int)sizeof(T));
}

struct GemmArgs {
    Hyper hy;
    const int32_t* tau;
    int M, N, K;                 // K in elements (the loop runs over round_up(K, k per tile))
    // P operand: base + it*p_it + g*p_g, rows of ldp elements; or (gather) the minibatch rows
    // of the group's shard, selected by idx / the cyclic window
    const void* P; int64_t p_it, p_g; int ldp; int gather;
    // Q operand: either per (it,g) like P, or a weight copy indexed by ring slot
    const void* Q; int64_t q_it, q_g, q_slot; int ldq; int q_is_weight;
    // FWD : bias from the fp32 ring (offset boff), outputs A [M][ldo] and AT [N][ldt]
    // DA  : ReLU mask from relu_bits (written by the FWD launch of that layer), outputs dZ and dZT
    // HEAD: output layer (N = classes <= 128, one tile holds whole rows): bias, softmax
    //       cross-entropy against the labels, outputs dZ_L and dZ_L^T, one loss partial per block
    const float* ring; int64_t boff;
    // one bit per element of a hidden layer's output, "activation > 0", in the accumulator layout
    // of the tile that produced it: word [(it*G + g), tile row, tile column][i*TN + j][thread],
    // bit e.  FWD writes it, the DA launch with the same output shape (and tile shape) reads it
    uint16_t* relu_bits;
    void* O; int64_t o_it, o_g; int ldo;
    void* OT; int64_t t_it, t_g; int ldt;
    // DW : fresh gradient block -> grad[g*p + goff + m*N + n]; partial ||fresh-stale||^2
    float* gbuf; const int32_t* which; int64_t goff;
    double* part_stat; int n_stat; int stat_off;
    int G;
    // HEAD
    const ShardDesc* shards; const int32_t* idx; double* part_loss;
    // DW: when given, the fresh gradient block of group g is written only if store_now[g] != 0
    // (the statistic is computed either way)
    const uint8_t* store_now;
    // DA: when given, the transposed output of group g is written only if t_flags[g] != 0
    // (first-layer signal under the Gram statistic: only a group that uploads needs it, for its
    // weight gradient; the others get it from mlp_gather_vec if they are selected after all)
    const uint8_t* t_flags;
};

template <typename T>
__device__ __forceinline__ void mfma_step(const uint4& a, const uint4& b, f32x16& acc);

template <>
__device__ __forceinline__ void mfma_step<bf16_t>(const uint4& a, const uint4& b, f32x16& acc)
{
    bf16x8 av, bv;
    __builtin_memcpy(&av, &a, 16);
    __builtin_memcpy(&bv, &b, 16);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc, 0, 0, 0);
}

template <>
__device__ __forceinline__ void mfma_step<float>(const uint4& a, const uint4& b, f32x16& acc)
{
    // four k-pairs; the k index a lane half contributes is the same for both operands
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
}

// A 16-byte load that is known to come from global memory.  The operand pointers may derive from
// the shard table (read from memory), whose address space the compiler cannot see: it would
// issue FLAT loads, and those are also counted with the LDS traffic -- every wait for an LDS
// fragment would then wait for the tile loads in flight as well.
__device__ __forceinline__ u32x4 global_load_vec(const char* p)
{
    return *(const __attribute__((address_space(1))) u32x4*)p;
}

// global -> registers: the 16-byte chunks of one k-tile of both operands.  (Native vector
// registers: arrays of the HIP uint4 struct are not always kept in registers.)
template <typename TL>
__device__ __forceinline__ void tile_gload(const char* __restrict__ Pg, const char* __restrict__ Qg,
                                           const int64_t (&poff)[TL::PCH], int64_t ldq_b, int kt,
                                           u32x4 (&rp)[TL::PCH], u32x4 (&rq)[TL::QCH])
{
    const int tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < TL::PCH; ++i) {
        const int kc = (tid + TL::NT * i) % TL::CPR;
        rp[i] = global_load_vec(Pg + poff[i] + (int64_t)kt * TL::KROW + kc * 16);
    }
#pragma unroll
    for (int i = 0; i < TL::QCH; ++i) {
        const int c = tid + TL::NT * i, row = c / TL::CPR, kc = c % TL::CPR;
        rq[i] = global_load_vec(Qg + (int64_t)row * ldq_b + (int64_t)kt * TL::KROW + kc * 16);
    }
}

template <typename TL>
__device__ __forceinline__ void tile_lstore(char* lp, char* lq, const u32x4 (&rp)[TL::PCH],
                                            const u32x4 (&rq)[TL::QCH])
{
    const int tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < TL::PCH; ++i) {
        const int c = tid + TL::NT * i, row = c / TL::CPR, kc = c % TL::CPR;
        *(u32x4*)(lp + row * TL::PITCH + kc * 16) = rp[i];
    }
#pragma unroll
    for (int i = 0; i < TL::QCH; ++i) {
        const int c = tid + TL::NT * i, row = c / TL::CPR, kc = c % TL::CPR;
        *(u32x4*)(lq + row * TL::PITCH + kc * 16) = rq[i];
    }
}

template <typename T, typename TL>
__device__ __forceinline__ void tile_mma(const char* lp, const char* lq, f32x16 (&acc)[TL::TM][TL::TN])
{
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int wm = wave / TL::WN, wn = wave % TL::WN;
    const int half = lane >> 5, r = lane & 31;
#pragma unroll
    for (int ks = 0; ks < TL::KS; ++ks) {
        uint4 a[TL::TM], b[TL::TN];
#pragma unroll
        for (int i = 0; i < TL::TM; ++i)
            a[i] = *(const uint4*)(lp + (wm * (TL::BM / TL::WM) + i * 32 + r) * TL::PITCH + ks * 32 + half * 16);
#pragma unroll
        for (int j = 0; j < TL::TN; ++j)
            b[j] = *(const uint4*)(lq + (wn * (TL::BN / TL::WN) + j * 32 + r) * TL::PITCH + ks * 32 + half * 16);
#pragma unroll
        for (int i = 0; i < TL::TM; ++i)
#pragma unroll
            for (int j = 0; j < TL::TN; ++j) mfma_step<T>(a[i], b[j], acc[i][j]);
    }
}

// One pass of the k-loop for a tile: acc += P_tile Q_tile^T.  Two LDS stages.  PF = 1: the next
// k-tile travels global -> registers while the current one is multiplied.  PF = 2: two k-tiles
// are in flight in two register sets, which covers the load latency when the multiply of one
// k-tile is shorter than a trip to L2 / HBM.  Loads past the last k-tile repeat the last one.
template <typename T, typename TL>
__device__ __forceinline__ void gemm_mainloop(const char* __restrict__ Pg, const char* __restrict__ Qg,
                                              const int64_t (&poff)[TL::PCH], int64_t ldq_b, int K, char* lds,
                                              f32x16 (&acc)[TL::TM][TL::TN])
{
    constexpr int kElemsPerTileK = TL::KROW / (int)sizeof(T);
    constexpr int kP = TL::BM * TL::PITCH;
    const int nk = (K + kElemsPerTileK - 1) / kElemsPerTileK;
    if constexpr (TL::PF == 1) {
        u32x4 rp[TL::PCH], rq[TL::QCH];
        tile_gload<TL>(Pg, Qg, poff, ldq_b, 0, rp, rq);
        tile_lstore<TL>(lds, lds + kP, rp, rq);
        __syncthreads();
        for (int kt = 0; kt + 1 < nk; ++kt) {
            char* cur = lds + (kt & 1) * TL::STAGE;
            char* nxt = lds + ((kt + 1) & 1) * TL::STAGE;
            tile_gload<TL>(Pg, Qg, poff, ldq_b, kt + 1, rp, rq);
            tile_mma<T, TL>(cur, cur + kP, acc);
            tile_lstore<TL>(nxt, nxt + kP, rp, rq);
            __syncthreads();
        }
        {
            const char* cur = lds + ((nk - 1) & 1) * TL::STAGE;
            tile_mma<T, TL>(cur, cur + kP, acc);
            __syncthreads();
        }
    } else {
        u32x4 rp0[TL::PCH], rq0[TL::QCH], rp1[TL::PCH], rq1[TL::QCH];
        const int last = nk - 1;
        tile_gload<TL>(Pg, Qg, poff, ldq_b, 0, rp0, rq0);
        tile_gload<TL>(Pg, Qg, poff, ldq_b, last < 1 ? last : 1, rp1, rq1);
        tile_lstore<TL>(lds, lds + kP, rp0, rq0);
        __syncthreads();
        // iteration kt: request tile kt+2 into the set tile kt came from, multiply tile kt,
        // move tile kt+1 from its set to the other LDS stage
        for (int kt = 0; kt < nk; kt += 2) {
            {
                char* cur = lds;
                char* nxt = lds + TL::STAGE;
                tile_gload<TL>(Pg, Qg, poff, ldq_b, kt + 2 < last ? kt + 2 : last, rp0, rq0);
                tile_mma<T, TL>(cur, cur + kP, acc);
                tile_lstore<TL>(nxt, nxt + kP, rp1, rq1);
                __syncthreads();
            }
            if (kt + 1 < nk) {
                char* cur = lds + TL::STAGE;
                char* nxt = lds;
                tile_gload<TL>(Pg, Qg, poff, ldq_b, kt + 3 < last ? kt + 3 : last, rp1, rq1);
                tile_mma<T, TL>(cur, cur + kP, acc);
                tile_lstore<TL>(nxt, nxt + kP, rp0, rq0);
                __syncthreads();
            }
        }
    }
}

// Weight gradients: the fresh gradient block of a tile goes to gbuf[fresh row of g][goff + m*N + n].
// accumulator element e of a lane: column n = lane % 32, row m = (e/4)*8 + (lane/32)*4 + e%4
template <typename TL>
__device__ __forceinline__ void dw_store_fresh(const GemmArgs& a, int g, int m0, int n0,
                                               const f32x16 (&acc)[TL::TM][TL::TN])
{
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int wm = wave / TL::WN, wn = wave % TL::WN;
    constexpr int RW = TL::BM / TL::WM, CW = TL::BN / TL::WN;
    const int cl = lane & 31, rh = (lane >> 5) * 4;
    float* gb = fresh_row(a.gbuf, a.which, a.hy, g) + a.goff;
    if (m0 + TL::BM <= a.M && n0 + TL::BN <= a.N) {
        // tile inside the matrix (the usual case): no bounds checks.  The row address is the
        // same for the whole wave (scalar registers); a lane adds one 32-bit byte offset, the
        // column block is an immediate
        const int uw = __builtin_amdgcn_readfirstlane(wave);
        char* wb = (char*)(gb + (int64_t)(m0 + (uw / TL::WN) * RW) * a.N + (n0 + (uw % TL::WN) * CW));
        const unsigned lo4 = (unsigned)(rh * a.N + cl) * 4u;
#pragma unroll
        for (int i = 0; i < TL::TM; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                char* rowb = wb + (int64_t)(i * 32 + (e >> 2) * 8 + (e & 3)) * a.N * 4;
#pragma unroll
                for (int j = 0; j < TL::TN; ++j) *(float*)(rowb + (lo4 + (unsigned)j * 128u)) = acc[i][j][e];
            }
        return;
    }
#pragma unroll
    for (int i = 0; i < TL::TM; ++i)
#pragma unroll
        for (int j = 0; j < TL::TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + wm * RW + i * 32 + (e >> 2) * 8 + rh + (e & 3);
                const int n = n0 + wn * CW + j * 32 + cl;
                if (m < a.M && n < a.N) gb[(int64_t)m * a.N + n] = acc[i][j][e];
            }
}

// k-tile t of two passes laid end to end: tiles 0..nk-1 from (Pg, Qg), tiles nk..2nk-1 from the
// same places dP / dQ bytes further on
template <typename TL>
__device__ __forceinline__ void tile_gload2(const char* __restrict__ Pg, const char* __restrict__ Qg,
                                            const int64_t (&poff)[TL::PCH], int64_t ldq_b, int64_t dP,
                                            int64_t dQ, int nk, int t, u32x4 (&rp)[TL::PCH],
                                            u32x4 (&rq)[TL::QCH])
{
    const bool second = t >= nk;
    tile_gload<TL>(Pg + (second ? dP : 0), Qg + (second ? dQ : 0), poff, ldq_b, second ? t - nk : t, rp, rq);
}

// The weight-gradient k-loops of both iterates as ONE software pipeline (PF = 2 only): with K =
// the minibatch size a pass is a handful of k-tiles, and two separate passes would fill and
// drain the pipeline twice.  Between the last tile of the first pass and the first tile of the
// second the accumulators hold the fresh block, which is stored there -- the stores drain while
// the second pass runs.  The number of k-tiles per pass must be even (a turn of the loop handles
// two tiles and the store sits between two turns).
// One turn of the two-passes loop: k-tiles kt and kt+1 (kt even).  Requests tiles kt+2 and kt+3
// (clamped to the last one) into the register sets, multiplies kt and kt+1 from the LDS stages.
template <typename T, typename TL>
__device__ __forceinline__ void two_passes_turn(const char* __restrict__ Pg, const char* __restrict__ Qg,
                                                const int64_t (&poff)[TL::PCH], int64_t ldq_b, int64_t dP,
                                                int64_t dQ, int nk, int kt, int last, char* lds,
                                                u32x4 (&rp0)[TL::PCH], u32x4 (&rq0)[TL::QCH],
                                                u32x4 (&rp1)[TL::PCH], u32x4 (&rq1)[TL::QCH],
                                                f32x16 (&acc)[TL::TM][TL::TN])
{
    constexpr int kP = TL::BM * TL::PITCH;
    {
        char* cur = lds;
        char* nxt = lds + TL::STAGE;
        tile_gload2<TL>(Pg, Qg, poff, ldq_b, dP, dQ, nk, kt + 2 < last ? kt + 2 : last, rp0, rq0);
        tile_mma<T, TL>(cur, cur + kP, acc);
        tile_lstore<TL>(nxt, nxt + kP, rp1, rq1);
        __syncthreads();
    }
    {
        char* cur = lds + TL::STAGE;
        char* nxt = lds;
        tile_gload2<TL>(Pg, Qg, poff, ldq_b, dP, dQ, nk, kt + 3 < last ? kt + 3 : last, rp1, rq1);
        tile_mma<T, TL>(cur, cur + kP, acc);
        tile_lstore<TL>(nxt, nxt + kP, rp0, rq0);
        __syncthreads();
    }
}

template <typename T, typename TL>
__device__ __forceinline__ void gemm_mainloop_two_passes(
    const char* __restrict__ Pg, const char* __restrict__ Qg, const int64_t (&poff)[TL::PCH],
    int64_t ldq_b, int64_t dP, int64_t dQ, int K, char* lds, f32x16 (&acc)[TL::TM][TL::TN],
    const GemmArgs& a, int g, int m0, int n0)
{
    static_assert(TL::PF == 2, "two k-tiles in flight");
    constexpr int kElemsPerTileK = TL::KROW / (int)sizeof(T);
    constexpr int kP = TL::BM * TL::PITCH;
    const int nk = (K + kElemsPerTileK - 1) / kElemsPerTileK;     // even
    const int total = 2 * nk, last = total - 1;
    u32x4 rp0[TL::PCH], rq0[TL::QCH], rp1[TL::PCH], rq1[TL::QCH];
    tile_gload2<TL>(Pg, Qg, poff, ldq_b, dP, dQ, nk, 0, rp0, rq0);
    tile_gload2<TL>(Pg, Qg, poff, ldq_b, dP, dQ, nk, 1, rp1, rq1);
    tile_lstore<TL>(lds, lds + kP, rp0, rq0);
    __syncthreads();
    // first pass; its last turn already requests the first tiles of the second
    for (int kt = 0; kt < nk; kt += 2)
        two_passes_turn<T, TL>(Pg, Qg, poff, ldq_b, dP, dQ, nk, kt, last, lds, rp0, rq0, rp1, rq1, acc);
    if (!a.store_now || a.store_now[g]) dw_store_fresh<TL>(a, g, m0, n0, acc);
    for (int kt = nk; kt < total; kt += 2)
        two_passes_turn<T, TL>(Pg, Qg, poff, ldq_b, dP, dQ, nk, kt, last, lds, rp0, rq0, rp1, rq1, acc);
}

__device__ __forceinline__ int stale_slot(const Hyper& hy, const int32_t* tau, int g)
{
    return stale_slot_of(hy, tau[g]);
}

// acc += P Q^T over the whole k range, operands of iterate `it` (0: theta^k, 1: the group's
// stale iterate) of group g, tile origin (m0, n0)
template <typename T, typename TL>
__device__ __forceinline__ void gemm_pass(const GemmArgs& a, int it, int g, int m0, int n0, char* lds,
                                          f32x16 (&acc)[TL::TM][TL::TN])
{
    constexpr int esz = (int)sizeof(T);
    // byte offset of the P row each of this thread's chunks belongs to: rows of the operand
    // array, or -- first layer -- the minibatch rows of the group's shard, read in place
    const char* Pg;
    int64_t poff[TL::PCH];
    if (a.gather) {
        const ShardDesc sh = a.shards[g];
        Pg = (const char*)sh.X;
#pragma unroll
        for (int i = 0; i < TL::PCH; ++i) {
            const int m = m0 + (threadIdx.x + TL::NT * i) / TL::CPR;
            int64_t row = 0;                     // rows past the minibatch: any valid row, result unused
            if (m < a.M) {
                if (a.idx) row = a.idx[(int64_t)g * a.hy.mu + m];
                else row = (int64_t)(((unsigned long long)a.hy.k * (unsigned long long)a.hy.mu +
                                      (unsigned long long)m) % (unsigned long long)sh.rows);
            }
            poff[i] = row * sh.ld * esz;
        }
    } else {
        Pg = (const char*)a.P + ((int64_t)it * a.p_it + (int64_t)g * a.p_g + (int64_t)m0 * a.ldp) * esz;
#pragma unroll
        for (int i = 0; i < TL::PCH; ++i)
            poff[i] = (int64_t)((threadIdx.x + TL::NT * i) / TL::CPR) * a.ldp * esz;
    }
    const char* Qg;
    if (a.q_is_weight) {
        const int slot = it == 0 ? a.hy.cur : stale_slot(a.hy, a.tau, g);
        Qg = (const char*)a.Q + ((int64_t)slot * a.q_slot + (int64_t)n0 * a.ldq) * esz;
    } else {
        Qg = (const char*)a.Q + ((int64_t)it * a.q_it + (int64_t)g * a.q_g + (int64_t)n0 * a.ldq) * esz;
    }
    gemm_mainloop<T, TL>(Pg, Qg, poff, (int64_t)a.ldq * esz, a.K, lds, acc);
}

// A 16-byte chunk of row `row` of the transposed staging tile.  Two-byte elements: the chunk's
// 8-byte halves are stored exchanged in every other group of eight rows (see the writes).
template <int ESZ>
__device__ __forceinline__ uint4 staged_t(const void* p, int row)
{
    const uint4 v = *(const uint4*)p;
    if constexpr (ESZ == 2) {
        const bool sw = (((row >> 3) ^ (row >> 4)) & 1) != 0;
        return sw ? make_uint4(v.z, v.w, v.x, v.y) : v;
    } else {
        return v;
    }
}

// grid: (ceil(N/BN), ceil(M/BM), batch);  batch = 2G (it*G + g) for FWD / DA / HEAD, G for DW.
template <typename T, int EPI, typename TL>
__global__ __launch_bounds__(TL::NT, TL::WPE) void mlp_gemm(GemmArgs a)
{
    extern __shared__ __align__(16) char lds[];
    constexpr int BM = TL::BM, BN = TL::BN, TM = TL::TM, TN = TL::TN;
    const Hyper& hy = a.hy;
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    constexpr int kGemmThreads = TL::NT, RW = BM / TL::WM, CW = BN / TL::WN;   // rows, columns per wave
    const int wm = wave / TL::WN, wn = wave % TL::WN;
    // Workgroup -> (tile, group, iterate).  Consecutive workgroup ids go to different XCDs (id mod
    // 8), each with its own L2.  The ids of one XCD are therefore mapped to a contiguous range of
    // work, ordered so that neighbours share operands: for the weight gradients all tiles of a
    // group (its signals and activations stay in that L2); otherwise all groups of one
    // (iterate, column tile), which share the weight tile.
    int bx, by, g, it0;
    {
        const int nx = gridDim.x, ny = gridDim.y, total = nx * ny * gridDim.z;
        const int lin = blockIdx.x + nx * (blockIdx.y + ny * blockIdx.z);
        int l = total % 8 == 0 ? (lin % 8) * (total / 8) + lin / 8 : lin;
        if (EPI == EPI_DW) {
            bx = l % nx; l /= nx;
            by = l % ny;
            g = l / ny;
            it0 = 0;
        } else {
            g = l % a.G; l /= a.G;
            by = l % ny; l /= ny;
            bx = l % nx;
            it0 = l / nx;
        }
    }
    const int m0 = by * BM, n0 = bx * BN;
    // server-side rule: unselected groups evaluate nothing (their loss partial is zero), the
    // others one gradient at theta^k only
    if (hy.sel) {
        if (!hy.sel[g]) {
            if (EPI == EPI_HEAD && it0 == 0 && tid == 0) a.part_loss[(int64_t)g * gridDim.y + by] = 0;
            return;
        }
        if (EPI != EPI_DW && it0 == 1) return;
    }
    constexpr int esz = (int)sizeof(T);

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
    // accumulator element e of lane: column n = lane % 32, row m = (e/4)*8 + (lane/32)*4 + e%4
    const int cl = lane & 31, rh = (lane >> 5) * 4;

    if constexpr (EPI == EPI_DW) {
        // The transposed signal of the stale iterate is stored NEGATED by the kernel that
        // produces it.  So: multiply at theta^k, write the fresh gradient block, then keep
        // accumulating the stale products into the same registers, which then hold
        // fresh - stale -- one accumulator set serves both iterates, and the two k-loops run as
        // one pipeline (gemm_mainloop_two_passes).
        if (hy.sel) {                            // server-side rule: no stale pass, no statistic
            gemm_pass<T, TL>(a, 0, g, m0, n0, lds, acc);
            dw_store_fresh<TL>(a, g, m0, n0, acc);
            return;
        }
        constexpr int kTileK = TL::KROW / (int)sizeof(T);
        if (((a.K + kTileK - 1) / kTileK) % 2 != 0) {
            // odd number of k-tiles per pass: two pipelines
            gemm_pass<T, TL>(a, 0, g, m0, n0, lds, acc);
            if (!a.store_now || a.store_now[g]) dw_store_fresh<TL>(a, g, m0, n0, acc);
            gemm_pass<T, TL>(a, 1, g, m0, n0, lds, acc);
        } else {
            // both passes in one pipeline; the fresh block is stored between them
            const char* Pg = (const char*)a.P + ((int64_t)g * a.p_g + (int64_t)m0 * a.ldp) * esz;
            const char* Qg = (const char*)a.Q + ((int64_t)g * a.q_g + (int64_t)n0 * a.ldq) * esz;
            int64_t poff[TL::PCH];
#pragma unroll
            for (int i = 0; i < TL::PCH; ++i)
                poff[i] = (int64_t)((threadIdx.x + TL::NT * i) / TL::CPR) * a.ldp * esz;
            gemm_mainloop_two_passes<T, TL>(Pg, Qg, poff, (int64_t)a.ldq * esz, a.p_it * esz, a.q_it * esz,
                                            a.K, lds, acc, a, g, m0, n0);
        }
        double sq = 0;
        if (m0 + BM <= a.M && n0 + BN <= a.N) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const float df = acc[i][j][e];
                        sq += (double)df * (double)df;
                    }
        } else {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int m = m0 + wm * RW + i * 32 + (e >> 2) * 8 + rh + (e & 3);
                        const int n = n0 + wn * CW + j * 32 + cl;
                        if (m < a.M && n < a.N) {
                            const float df = acc[i][j][e];
                            sq += (double)df * (double)df;
                        }
                    }
        }
        sq = wave_sum(sq);
        double* red = (double*)lds;
        __syncthreads();
        if (lane == 0) red[wave] = sq;
        __syncthreads();
        if (tid == 0) {
            double t = 0;
#pragma unroll
            for (int wv = 0; wv < TL::NW; ++wv) t += red[wv];
            a.part_stat[(int64_t)g * a.n_stat + a.stat_off + by * gridDim.x + bx] = t;
        }
        return;
    }
    if constexpr (EPI == EPI_FWD) {
        // hidden layer: the accumulators start at the bias of their column (the load runs under
        // the first tile loads; the epilogue has one addition per element less)
        const int slot = it0 == 0 ? hy.cur : stale_slot(hy, a.tau, g);
        const float* bias = a.ring + (int64_t)slot * hy.pstride + a.boff;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = n0 + wn * CW + j * 32 + cl;
            const float bv = n < a.N ? round_to<T>(bias[n]) : 0.0f;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = bv;
        }
    }
    gemm_pass<T, TL>(a, it0, g, m0, n0, lds, acc);
    if constexpr (EPI == EPI_HEAD) {
        // logits tile -> LDS (fp32), then one thread per sample: softmax cross-entropy and dZ_L
        static_assert(BN <= kHeadClasses && BM <= TL::NT, "output-layer tile");
        constexpr int pitch = BN + 4;
        float* lg = (float*)lds;
        const int slot = it0 == 0 ? hy.cur : stale_slot(hy, a.tau, g);
        const float* bias = a.ring + (int64_t)slot * hy.pstride + a.boff;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int nl = wn * CW + j * 32 + cl;
                const float bv = nl < a.N ? round_to<T>(bias[nl]) : 0.0f;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int ml = wm * RW + i * 32 + (e >> 2) * 8 + rh + (e & 3);
                    lg[ml * pitch + nl] = acc[i][j][e] + bv;
                }
            }
        __syncthreads();
        T* O = (T*)a.O + (int64_t)it0 * a.o_it + (int64_t)g * a.o_g;        // dZ_L   [mu][ldo]
        T* OT = (T*)a.OT + (int64_t)it0 * a.t_it + (int64_t)g * a.t_g;      // dZ_L^T [N][ldt]
        double lsum = 0;
        const int nc = a.N;
        if (tid < BM && m0 + tid < a.M) {
            const int i = m0 + tid;
            const ShardDesc sh = a.shards[g];
            int64_t row;
            if (a.idx) row = a.idx[(int64_t)g * hy.mu + i];
            else row = (int64_t)(((unsigned long long)hy.k * (unsigned long long)hy.mu +
                                  (unsigned long long)i) % (unsigned long long)sh.rows);
            const int y = global_load((const int32_t*)sh.y + row);
            float* z = lg + tid * pitch;
            // Everything relative to the true class, so that a confidently right sample
            // (p_y -> 1) loses no digits: t_c = z_c - z_y, m = max_c t_c >= 0,
            // S = sum_c exp(t_c - m); loss = m + log S; p_c = exp(t_c - m) / S;
            // dZ_c = p_c (c != y), dZ_y = -sum_{c != y} p_c.
            const float zy = z[y];
            float m = 0.0f;
            for (int c = 0; c < nc; ++c) m = fmaxf(m, z[c] - zy);
            // (every exponent is <= 0: the hardware exponential with a corrected argument, a few
            // ulp, once per class)
            float so = 0.0f;
            for (int c = 0; c < nc; ++c)
                if (c != y) {
                    const float ev = exp_nonpos(z[c] - zy - m);
                    z[c] = ev;
                    so += ev;
                }
            const float ey = exp_nonpos(-m);
            const float inv = 1.0f / (ey + so);
            float others = 0.0f;
            for (int c = 0; c < nc; ++c) {
                if (c == y) continue;
                const float dv = z[c] * inv;
                others += dv;
                z[c] = dv;
            }
            z[y] = -others;
            lsum = m == 0.0f ? (double)log1pf(so) : (double)(m + logf(ey + so));
            for (int c = 0; c < nc; ++c) O[(int64_t)i * a.ldo + c] = to_T<T>(z[c]);
        } else if (tid < BM) {
            for (int c = 0; c < nc; ++c) lg[tid * pitch + c] = 0.0f;
        }
        lsum = wave_sum(lsum);
        __syncthreads();
        double* red = (double*)(lg + BM * pitch);
        if (lane == 0) red[wave] = lsum;
        // transposed copy: class c, samples m0 .. m0+BM-1 (zeros beyond M keep the padding clean);
        // negated for the stale iterate (the weight-gradient kernel subtracts by accumulating)
        const float tsign = it0 == 1 ? -1.0f : 1.0f;
        constexpr int V = 16 / esz;
        for (int c2 = tid; c2 < nc * (BM / V); c2 += kGemmThreads) {
            const int c = c2 / (BM / V), mv = (c2 % (BM / V)) * V;
            if (m0 + mv < a.M) {
                alignas(16) T tmp[V];
#pragma unroll
                for (int q = 0; q < V; ++q) tmp[q] = to_T<T>(tsign * lg[(mv + q) * pitch + c]);
                *(uint4*)(OT + (int64_t)c * a.ldt + m0 + mv) = *(const uint4*)tmp;
            }
        }
        __syncthreads();
        if (it0 == 0 && tid == 0) {
            double t = 0;
#pragma unroll
            for (int wv = 0; wv < TL::NW; ++wv) t += red[wv];
            a.part_loss[(int64_t)g * gridDim.y + by] = t;
        }
    } else {
        // Two outputs: row-major O [M][ldo] and transposed OT [N][ldt].  The tile goes through
        // LDS twice, each time in the orientation of the output, written from the accumulators
        // in packed form (four rows of a column are adjacent registers; two columns of a row are
        // adjacent lanes) and read back as 16-byte vectors along the output's rows.
        constexpr int V = 16 / esz;                 // elements per 16-byte vector
        constexpr int PT = BM + V, PR = BN + V;     // row pitches of the two staging tiles
        T* st = (T*)lds;
        const bool inside = m0 + BM <= a.M && n0 + BN <= a.N;
        if constexpr (EPI == EPI_FWD) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[i][j][e] = fmaxf(acc[i][j][e], 0.0f);
            // which units are active, for the backward pass
            uint16_t* rb = a.relu_bits + ((((int64_t)it0 * a.G + g) * gridDim.y + by) * gridDim.x + bx) *
                                             (int64_t)(TM * TN * kGemmThreads);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    // bit e = [accumulator e > 0]: a compare and an add-with-carry per element
                    // (b = 2b + carry, from the last element down)
                    unsigned b = 0;
#pragma unroll
                    for (int e = 15; e >= 0; --e)
                        asm("v_cmp_lt_f32 vcc, 0, %1\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc"
                            : "+v"(b) : "v"(acc[i][j][e]) : "vcc");
                    rb[(i * TN + j) * kGemmThreads + tid] = (uint16_t)b;
                }
        } else {
            // ReLU mask of the layer this signal belongs to: clear the accumulators of inactive units
            const uint16_t* rb = a.relu_bits + ((((int64_t)it0 * a.G + g) * gridDim.y + by) * gridDim.x + bx) *
                                                   (int64_t)(TM * TN * kGemmThreads);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const unsigned b = rb[(i * TN + j) * kGemmThreads + tid];
                    // bit e, spread over a word, ANDed onto the accumulator: two instructions
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int keep = (int)(b << (31 - e)) >> 31;
                        acc[i][j][e] = __int_as_float(__float_as_int(acc[i][j][e]) & keep);
                    }
                }
        }
        // two-byte outputs: round the accumulators once, to packed pairs (rows 0,1 and rows 2,3 of
        // each group of four), for both stagings
        constexpr int NPK = esz == 2 ? 8 : 1;
        unsigned pk[TM][TN][NPK];
        if constexpr (esz == 2) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int h = 0; h < 8; ++h) pk[i][j][h] = pack_bf16x2(acc[i][j][2 * h], acc[i][j][2 * h + 1]);
        }
        // ---- transposed: stT [BN][PT], element (n, m) ----
        // (all staging rows of a lane share bits 3 and 4 of the row index: those of the lane)
        static_assert(CW % 32 == 0, "staging rows of a lane differ by multiples of 32");
        [[maybe_unused]] const int t_swap = esz == 2 ? (((cl >> 3) ^ (cl >> 4)) & 1) * 4 : 0;
        if (EPI != EPI_DA || !a.t_flags || a.t_flags[g]) {        // (the same for the whole workgroup)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int nl = wn * CW + j * 32 + cl;
#pragma unroll
                for (int eg = 0; eg < 4; ++eg) {
                    const int ml = wm * RW + i * 32 + eg * 8 + rh;      // rows ml .. ml+3
                    if constexpr (esz == 2) {
                        // the two 8-byte halves of a 16-byte chunk change places in every other
                        // group of eight staging rows (t_swap): the 16 lanes an 8-byte LDS write
                        // serves at a time then fall into different banks
                        *(uint2*)(st + nl * PT + (ml ^ t_swap)) = make_uint2(pk[i][j][2 * eg], pk[i][j][2 * eg + 1]);
                    } else {
                        alignas(16) T q4[4];
#pragma unroll
                        for (int q = 0; q < 4; ++q) q4[q] = to_T<T>(acc[i][j][eg * 4 + q]);
                        *(uint4*)(st + nl * PT + ml) = *(const uint4*)q4;
                    }
                }
            }
        __syncthreads();
        {
            T* OT = (T*)a.OT + (int64_t)it0 * a.t_it + (int64_t)g * a.t_g;
            // the stale iterate's transposed signal is stored negated for the weight-gradient
            // kernel: flip the sign bits of the packed values
            constexpr unsigned kSigns = esz == 2 ? 0x80008000u : 0x80000000u;
            const unsigned flip = (EPI == EPI_DA && it0 == 1) ? kSigns : 0u;
            if (inside) {
                // tile inside the matrix: the staged values go out as they are
#pragma unroll 4
                for (int c = tid; c < BN * (BM / V); c += kGemmThreads) {
                    const int nl = c / (BM / V), mv = (c % (BM / V)) * V;
                    uint4 v = staged_t<esz>(st + nl * PT + mv, nl);
                    v.x ^= flip; v.y ^= flip; v.z ^= flip; v.w ^= flip;
                    *(uint4*)(OT + (int64_t)(n0 + nl) * a.ldt + (m0 + mv)) = v;
                }
            } else
            for (int c = tid; c < BN * (BM / V); c += kGemmThreads) {
                const int nl = c / (BM / V), mv = (c % (BM / V)) * V;
                const int n = n0 + nl, m = m0 + mv;
                if (n < a.N && m < a.M) {
                    alignas(16) T tmp[V];
                    *(uint4*)tmp = staged_t<esz>(st + nl * PT + mv, nl);
#pragma unroll
                    for (int q = 0; q < V; ++q) {
                        float v = (m + q < a.M) ? to_f<T>(tmp[q]) : 0.0f;
                        // the stale iterate's transposed signal is stored negated for the
                        // weight-gradient kernel
                        if (EPI == EPI_DA && it0 == 1) v = -v;
                        tmp[q] = to_T<T>(v);
                    }
                    *(uint4*)(OT + (int64_t)n * a.ldt + m) = *(const uint4*)tmp;
                }
            }
        }
        __syncthreads();
        }
        // ---- row-major: stR [BM][PR], element (m, n) ----
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int nl = wn * CW + j * 32 + cl;
#pragma unroll
                for (int eg = 0; eg < 4; ++eg) {
                    const int ml = wm * RW + i * 32 + eg * 8 + rh;
                    if constexpr (esz == 2) {
                        // rows 0,1 and rows 2,3 as two packed words; the lane pair (n, n^1) swaps
                        // one word so that each lane holds two columns of two rows
                        const unsigned w01 = pk[i][j][2 * eg], w23 = pk[i][j][2 * eg + 1];
                        const bool odd = (lane & 1) != 0;
                        const unsigned give = odd ? w01 : w23;
                        const unsigned got = (unsigned)__builtin_amdgcn_mov_dpp((int)give, 0xB1, 0xF, 0xF, true);
                        // even lane: rows 0,1 of columns (n, n+1); odd lane: rows 2,3 of (n-1, n)
                        const unsigned mine = odd ? w23 : w01;
                        const unsigned left = odd ? got : mine, right = odd ? mine : got;
                        const unsigned ra = (left & 0xffffu) | (right << 16);          // first row
                        const unsigned rb = (left >> 16) | (right & 0xffff0000u);      // second row
                        const int mr = ml + (odd ? 2 : 0), nc2 = nl & ~1;
                        *(unsigned*)(st + (mr + 0) * PR + nc2) = ra;
                        *(unsigned*)(st + (mr + 1) * PR + nc2) = rb;
                    } else {
#pragma unroll
                        for (int q = 0; q < 4; ++q) st[(ml + q) * PR + nl] = to_T<T>(acc[i][j][eg * 4 + q]);
                    }
                }
            }
        __syncthreads();
        {
            T* O = (T*)a.O + (int64_t)it0 * a.o_it + (int64_t)g * a.o_g;
            if (inside) {
#pragma unroll 4
                for (int c = tid; c < BM * (BN / V); c += kGemmThreads) {
                    const int ml = c / (BN / V), nv = (c % (BN / V)) * V;
                    *(uint4*)(O + (int64_t)(m0 + ml) * a.ldo + (n0 + nv)) = *(const uint4*)(st + ml * PR + nv);
                }
            } else
            for (int c = tid; c < BM * (BN / V); c += kGemmThreads) {
                const int ml = c / (BN / V), nv = (c % (BN / V)) * V;
                const int m = m0 + ml, n = n0 + nv;
                if (m < a.M && n < a.N) {
                    // ldo is a multiple of 64 and pads stay zero: mask the lanes beyond N
                    alignas(16) T tmp[V];
                    *(uint4*)tmp = *(const uint4*)(st + ml * PR + nv);
#pragma unroll
                    for (int q = 0; q < V; ++q)
                        if (!(n + q < a.N)) tmp[q] = to_T<T>(0.0f);
                    *(uint4*)(O + (int64_t)m * a.ldo + n) = *(const uint4*)tmp;
                }
            }
        }
    }
}

// The weight gradients at theta^k of selected groups, all layers in ONE launch (the second half
// of the lazy gradient store).  The first layer takes the groups of `sel_first`, the deeper ones
// those of `sel_rest`.  Most of the time nobody is selected, so the launch must cost little when
// it has nothing to do: a fixed grid of one workgroup per compute unit; every workgroup lists
// the selected groups (ascending, in LDS behind the GEMM stages) and walks over the jobs
// (group, tile) blockIdx.x, blockIdx.x + gridDim.x, ... -- consecutive jobs are tiles of one
// group, so the workgroups running at any time share a few groups' operands.
// dynamic LDS: the GEMM stages + 2 G two-byte group ids.
struct DwSelectedArgs {
    GemmArgs layer[GCADA_MAX_WIDTHS - 1];
    int tile_end[GCADA_MAX_WIDTHS - 1];    // running totals of the layers' tile counts
    int n_layers;
    const uint8_t* sel_first;
    const uint8_t* sel_rest;
};
static_assert(sizeof(DwSelectedArgs) <= 4096, "kernel arguments");

// ascending list of the groups with sel[g] != 0; called by one whole wave, returns their number
__device__ __forceinline__ int list_selected(const uint8_t* __restrict__ sel, int G, uint16_t* list)
{
    const int lane = threadIdx.x % kWave;
    int n = 0;
    for (int g0 = 0; g0 < G; g0 += kWave) {
        const int g = g0 + lane;
        const bool on = g < G && sel[g];
        const unsigned long long bal = __ballot(on);
        if (on) list[n + __popcll(bal & ((1ull << lane) - 1ull))] = (uint16_t)g;
        n += __popcll(bal);
    }
    return n;
}

template <typename T, typename TL>
__global__ __launch_bounds__(TL::NT, TL::WPE) void mlp_dw_selected(DwSelectedArgs s)
{
    extern __shared__ __align__(16) char lds[];
    __shared__ int s_n[2];
    const int G = s.layer[0].hy.G;
    uint16_t* first = (uint16_t*)(lds + gemm_lds_bytes<T, EPI_DW, TL>());
    uint16_t* rest = first + G;
    if (threadIdx.x < kWave) {
        const int n0 = list_selected(s.sel_first, G, first);
        const int n1 = list_selected(s.sel_rest, G, rest);
        if (threadIdx.x == 0) { s_n[0] = n0; s_n[1] = n1; }
    }
    __syncthreads();
    const int tiles_first = s.tile_end[0], tiles_rest = s.tile_end[s.n_layers - 1] - tiles_first;
    const int jobs_first = s_n[0] * tiles_first, jobs = jobs_first + s_n[1] * tiles_rest;
    for (int j = blockIdx.x; j < jobs; j += gridDim.x) {
        int g, tile, li = 0;
        if (j < jobs_first) {
            g = first[j / tiles_first];
            tile = j % tiles_first;
        } else {
            const int jj = j - jobs_first;
            g = rest[jj / tiles_rest];
            tile = tiles_first + jj % tiles_rest;
            li = 1;
            while (li + 1 < s.n_layers && tile >= s.tile_end[li]) ++li;
        }
        const GemmArgs& a = s.layer[li];
        const int t = tile - (li ? s.tile_end[li - 1] : 0);
        const int nx = (a.N + TL::BN - 1) / TL::BN;
        const int bx = t % nx, by = t / nx;
        const int m0 = by * TL::BM, n0 = bx * TL::BN;
        f32x16 acc[TL::TM][TL::TN];
#pragma unroll
        for (int i = 0; i < TL::TM; ++i)
#pragma unroll
            for (int jn = 0; jn < TL::TN; ++jn)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][jn][e] = 0.0f;
        gemm_pass<T, TL>(a, 0, g, m0, n0, lds, acc);     // (ends with a barrier: the stages are free again)
        dw_store_fresh<TL>(a, g, m0, n0, acc);
    }
}

// Tile shapes.  bf16: 256 x 256 tiles with eight waves and two k-tiles in flight for the forward
// and signal GEMMs and for the weight gradients (128 x 256 tiles with two workgroups per compute
// unit -- the seventh Tile parameter -- were measured slower), 64 x 128 for the output layer, whose
// k loop is a chain of memory round trips.
// fp32: square tiles with 32 floats of k.
// SMALL: fp32 problems whose 128 x 128 tiles would leave most of the device idle (fp32 MFMA is
// slow enough that a workgroup's k loop is arithmetic-bound) use 64 x 64 tiles instead.
template <typename T, int EPI, bool SMALL> struct TileOf;
template <int EPI> struct TileOf<float, EPI, false> { using type = Tile<128, 128, 128, 2, 2, 2>; };
template <int EPI> struct TileOf<float, EPI, true> { using type = Tile<64, 64, 128, 2, 2, 2>; };
template <> struct TileOf<float, EPI_HEAD, true> { using type = Tile<64, 128, 128, 2, 2, 2>; };
// (fp32 MFMA is slow enough that a wave's 32 x 32 block is arithmetic-bound by itself: the weight
// gradients of small problems take 32 x 64 tiles, whose finer grain leaves fewer SIMDs with one
// block more than the others -- 784-200 at G = 10: 54 -> 48 us)
template <> struct TileOf<float, EPI_DW, true> { using type = Tile<32, 64, 128, 1, 2, 2>; };
template <bool SMALL> struct TileOf<bf16_t, EPI_FWD, SMALL> { using type = Tile<256, 256, 128, 4, 2, 2>; };
template <bool SMALL> struct TileOf<bf16_t, EPI_DA, SMALL> { using type = Tile<256, 256, 128, 4, 2, 2>; };
template <bool SMALL> struct TileOf<bf16_t, EPI_DW, SMALL> { using type = Tile<256, 256, 64, 4, 2, 2>; };
template <bool SMALL> struct TileOf<bf16_t, EPI_HEAD, SMALL> { using type = Tile<64, 128, 128, 2, 2, 2>; };

// Output layers of at most 32 classes (the usual case: ten) take a tile 32 columns wide instead
// of 128: a quarter of the weight rows to load, of the MFMA work and of the staging, and k-tiles
// twice as long (half the barriers of a loop that is a chain of memory round trips).
template <typename T> struct HeadNarrow { using type = Tile<64, 32, 256, 2, 1, 2>; };

// Weight gradients of a bf16 layer with at most 32 units (the output layer): 32 x 128 tiles
// instead of 256 x 256 ones whose rows would be padding, with k-tiles twice as long.
struct DwNarrow { using type = Tile<32, 128, 128, 1, 4, 2>; };
template <typename T> static bool dw_narrow(int M) { return sizeof(T) == 2 && M <= DwNarrow::type::BM; }

template <typename T, int EPI, typename TL>
static hipError_t launch_tile(const GemmArgs& a, int batch, hipStream_t s)
{
    constexpr int lds = gemm_lds_bytes<T, EPI, TL>();
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)mlp_gemm<T, EPI, TL>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((a.N + TL::BN - 1) / TL::BN, (a.M + TL::BM - 1) / TL::BM, batch);
    mlp_gemm<T, EPI, TL><<<grid, TL::NT, lds, s>>>(a);
    return hipGetLastError();
}

template <typename T, int EPI>
static hipError_t launch_gemm(const GemmArgs& a, int batch, bool small, hipStream_t s)
{
    if constexpr (EPI == EPI_HEAD) {
        using TN = typename HeadNarrow<T>::type;
        // (its longer k-tiles must end where the padded rows end; where they do not, the wide
        // tile has the same rows per workgroup, so the loss partials keep their places)
        static_assert(sizeof(T) == 4 || TN::BM == TileOf<T, EPI_HEAD, false>::type::BM, "loss partials");
        if (a.N <= TN::BN && (a.ldp * (int)sizeof(T)) % TN::KROW == 0 && (a.ldq * (int)sizeof(T)) % TN::KROW == 0) return launch_tile<T, EPI, TN>(a, batch, s);
    }
    if constexpr (EPI == EPI_DW && sizeof(T) == 2) {
        // (the padded minibatch length is a multiple of 64 elements = its k-tile)
        if (dw_narrow<T>(a.M)) return launch_tile<T, EPI, DwNarrow::type>(a, batch, s);
    }
    return small ? launch_tile<T, EPI, typename TileOf<T, EPI, true>::type>(a, batch, s)
                 : launch_tile<T, EPI, typename TileOf<T, EPI, false>::type>(a, batch, s);
}

// The narrow weight-gradient kernel (mlp_dw_narrow) serves a layer of a small fp32 model that
// has at most 16 outputs and a row-major activation to read (l >= 2).
static bool dw_narrow_layer(bool bf16, bool small, int l, int n_out)
{
    return !bf16 && small && l >= 2 && n_out <= 16;
}
// workgroups (statistic partials) of the weight-gradient GEMM of an M x N layer
template <typename T>
static int dw_blocks(int M, int N, bool small)
{
    using TB = typename TileOf<T, EPI_DW, false>::type;
    using TS = typename TileOf<T, EPI_DW, true>::type;
    using TN = DwNarrow::type;
    if (dw_narrow<T>(M)) return ((M + TN::BM - 1) / TN::BM) * ((N + TN::BN - 1) / TN::BN);
    return small ? ((M + TS::BM - 1) / TS::BM) * ((N + TS::BN - 1) / TS::BN)
                 : ((M + TB::BM - 1) / TB::BM) * ((N + TB::BN - 1) / TB::BN);
}
template <typename T>
static int head_row_blocks(int mu, bool small, int classes)
{
    using TB = typename TileOf<T, EPI_HEAD, false>::type;
    using TS = typename TileOf<T, EPI_HEAD, true>::type;
    using TN = typename HeadNarrow<T>::type;
    if (classes <= TN::BN) return (mu + TN::BM - 1) / TN::BM;
    return small ? (mu + TS::BM - 1) / TS::BM : (mu + TB::BM - 1) / TB::BM;
}

// ---------------------------------------------------------------------------------------
// Gather the minibatch rows of every group: Xg [G][mu][ld0] and its transpose XgT [G][n0][ldmu].
// grid: (ceil(n0/64), ceil(mu/64), G), block 256.
template <typename T>
__global__ __launch_bounds__(256) void mlp_gather(Hyper hy, const ShardDesc* __restrict__ shards,
                                                  const int32_t* __restrict__ idx, int n0, int ld0,
                                                  int ldmu, T* __restrict__ Xg, T* __restrict__ XgT)
{
    __shared__ T tile[64][64 + 2];
    const int g = blockIdx.z, c0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
    if (hy.sel && !hy.sel[g]) return;            // unselected group (server-side rule)
    const ShardDesc sh = shards[g];
    const T* X = (const T*)sh.X;
    const int tx = threadIdx.x % 64, ty = threadIdx.x / 64;
    for (int r = ty; r < 64; r += 4) {
        const int i = r0 + r;
        T v = to_T<T>(0.0f);
        if (i < hy.mu && c0 + tx < n0) {
            int64_t row;
            if (idx) row = idx[(int64_t)g * hy.mu + i];
            else row = (int64_t)(((unsigned long long)hy.k * (unsigned long long)hy.mu +
                                  (unsigned long long)i) % (unsigned long long)sh.rows);
            v = global_load(X + row * sh.ld + c0 + tx);
            Xg[((int64_t)g * hy.mu + i) * ld0 + c0 + tx] = v;
        }
        tile[r][tx] = v;
    }
    __syncthreads();
    for (int c = ty; c < 64; c += 4) {
        const int n = c0 + c, i = r0 + tx;
        if (n < n0 && i < hy.mu) XgT[((int64_t)g * n0 + n) * ldmu + i] = tile[tx][c];
    }
}

// The same with 16-byte accesses, for shards whose rows are 16-byte aligned and whose width is a
// multiple of the vector length.  Xg may be null (the first forward GEMM then reads the shard
// rows in place) -- only the transpose is written.
// grid: (ceil(n0 / (8 V)), ceil(mu/64), G), block 256; V = elements per 16 bytes.
// A second job of the same launch (workgroups with blockIdx.x >= the gather's ceil(n0 / TC)):
// the transpose of a dense per-group matrix D [G][mu][ldd] (nd columns) into DT [G][nd][ldmu], for
// the groups of `dsel` -- the first-layer signal of groups that are selected without having
// written its transposed copy in the gradient stage.
template <typename T>
struct DenseTranspose {
    const T* D;
    T* DT;
    int nd, ldd;
    const uint8_t* dsel;
};

template <typename T>
__global__ __launch_bounds__(256) void mlp_gather_vec(Hyper hy, const ShardDesc* __restrict__ shards,
                                                      const int32_t* __restrict__ idx, int n0, int ld0,
                                                      int ldmu, T* __restrict__ Xg, T* __restrict__ XgT,
                                                      DenseTranspose<T> dt)
{
    constexpr int V = 16 / (int)sizeof(T), TC = 8 * V, PITCH = 64 + V;
    __shared__ __align__(16) T tileT[TC][PITCH];
    const int g = blockIdx.z, r0 = blockIdx.y * 64;
    const int nbx = (n0 + TC - 1) / TC;
    if ((int)blockIdx.x >= nbx) {
        if (!dt.dsel[g]) return;
        const int c0 = ((int)blockIdx.x - nbx) * TC;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int t = threadIdx.x + 256 * h, r = t / 8, cv = (t % 8) * V;
            const int i = r0 + r, col = c0 + cv;
            alignas(16) T v[V];
#pragma unroll
            for (int q = 0; q < V; ++q) v[q] = to_T<T>(0.0f);
            // (rows are padded to ldd >= nd with zeros; ldd is a multiple of 64 elements)
            if (i < hy.mu && col < dt.ldd) *(uint4*)v = *(const uint4*)(dt.D + ((int64_t)g * hy.mu + i) * dt.ldd + col);
#pragma unroll
            for (int q = 0; q < V; ++q) tileT[cv + q][r] = v[q];
        }
        __syncthreads();
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int t = threadIdx.x + 256 * h, c = t / (64 / V), rv = (t % (64 / V)) * V;
            const int n = c0 + c, i = r0 + rv;
            if (n < dt.nd && i < hy.mu)
                *(uint4*)(dt.DT + ((int64_t)g * dt.nd + n) * ldmu + i) = *(const uint4*)&tileT[c][rv];
        }
        return;
    }
    const int c0 = blockIdx.x * TC;
    if (hy.sel && !hy.sel[g]) return;            // unselected group (server-side rule)
    const ShardDesc sh = shards[g];
    const T* X = (const T*)sh.X;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int t = threadIdx.x + 256 * h, r = t / 8, cv = (t % 8) * V;
        const int i = r0 + r, col = c0 + cv;
        alignas(16) T v[V];
#pragma unroll
        for (int q = 0; q < V; ++q) v[q] = to_T<T>(0.0f);
        if (i < hy.mu && col < n0) {
            int64_t row;
            if (idx) row = idx[(int64_t)g * hy.mu + i];
            else row = (int64_t)(((unsigned long long)hy.k * (unsigned long long)hy.mu +
                                  (unsigned long long)i) % (unsigned long long)sh.rows);
            *(u32x4*)v = global_load_vec((const char*)(X + row * sh.ld + col));
            if (Xg) *(uint4*)(Xg + ((int64_t)g * hy.mu + i) * ld0 + col) = *(const uint4*)v;
        }
#pragma unroll
        for (int q = 0; q < V; ++q) tileT[cv + q][r] = v[q];
    }
    __syncthreads();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int t = threadIdx.x + 256 * h, c = t / (64 / V), rv = (t % (64 / V)) * V;
        const int n = c0 + c, i = r0 + rv;
        if (n < n0 && i < hy.mu)
            *(uint4*)(XgT + ((int64_t)g * n0 + n) * ldmu + i) = *(const uint4*)&tileT[c][rv];
    }
}

// Compute copies of the hidden-layer weights of one ring slot: Wc [n_l][ld_{l-1}] and the
// transpose WcT [n_{l-1}][ld_l], both in T.  One 64 x 64 block of a layer: (bx, by) of
// (ceil(n_in/64), ceil(n_out/64)); 256 threads.
template <typename T>
__device__ __forceinline__ void weight_copy_block(int bx, int by, const float* __restrict__ W, int n_out,
                                                  int n_in, int ld_in, int ld_out, T* __restrict__ Wc,
                                                  T* __restrict__ WcT)
{
    __shared__ T tile[64][64 + 2];
    const int i0 = bx * 64, o0 = by * 64;
    const int tx = threadIdx.x % 64, ty = threadIdx.x / 64;
    for (int r = ty; r < 64; r += 4) {
        const int o = o0 + r, i = i0 + tx;
        T v = to_T<T>(0.0f);
        if (o < n_out && i < n_in) {
            v = to_T<T>(W[(int64_t)o * n_in + i]);
            Wc[(int64_t)o * ld_in + i] = v;
        }
        tile[r][tx] = v;
    }
    __syncthreads();
    for (int c = ty; c < 64; c += 4) {
        const int i = i0 + c, o = o0 + tx;
        if (WcT && i < n_in && o < n_out) WcT[(int64_t)i * ld_out + o] = tile[tx][c];
    }
}

// The same with 16-byte loads and 8/16-byte stores, for layers whose input width is a multiple
// of 4 and whose weights start 16-byte aligned in the parameter vector.  WcT may be null (the
// first layer's transpose is never used: no signal is propagated to the input).
template <typename T>
__device__ __forceinline__ void weight_copy_block_vec(int bx, int by, const float* __restrict__ W, int n_out,
                                                      int n_in, int ld_in, int ld_out, T* __restrict__ Wc,
                                                      T* __restrict__ WcT)
{
    constexpr int V = 16 / (int)sizeof(T), PITCH = 64 + 8;
    __shared__ __align__(16) T tileT[64][PITCH];
    const int i0 = bx * 64, o0 = by * 64;
#pragma unroll
    for (int h = 0; h < 4; ++h) {
        const int t = threadIdx.x + 256 * h, r = t / 16, cv = (t % 16) * 4;
        const int o = o0 + r, i = i0 + cv;
        alignas(16) T v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = to_T<T>(0.0f);
        if (o < n_out && i < n_in) {
            const float4 w4 = *(const float4*)(W + (int64_t)o * n_in + i);
            v[0] = to_T<T>(w4.x); v[1] = to_T<T>(w4.y); v[2] = to_T<T>(w4.z); v[3] = to_T<T>(w4.w);
            if constexpr (sizeof(T) == 2) *(uint2*)(Wc + (int64_t)o * ld_in + i) = *(const uint2*)v;
            else *(uint4*)(Wc + (int64_t)o * ld_in + i) = *(const uint4*)v;
        }
        if (WcT) {
#pragma unroll
            for (int q = 0; q < 4; ++q) tileT[cv + q][r] = v[q];
        }
    }
    if (!WcT) return;
    __syncthreads();
    constexpr int NV = 64 / V;                    // 16-byte vectors per transposed row
    for (int t = threadIdx.x; t < 64 * NV; t += 256) {
        const int c = t / NV, rv = (t % NV) * V;
        const int i = i0 + c, o = o0 + rv;
        // columns past n_out up to the padded row length receive the zeros they must hold
        if (i < n_in && o < ld_out) *(uint4*)(WcT + (int64_t)i * ld_out + o) = *(const uint4*)&tileT[c][rv];
    }
}

// The copies of all layers of one ring slot in ONE launch (a launch costs more than a small
// layer's copy), and in its last workgroup, when `store_now` is given, the store flags of the
// lazy gradient store for the step that follows (they depend on the ages and the history the
// server step has just written).
// grid: (blocks of all layers together + 1), block 256.
struct RefreshArgs {
    struct LayerCopy {
        const float* W;
        void* Wc;
        void* WcT;
        int n_out, n_in, ld_in, ld_out;
        int nbx;           // blocks along the input width
        int block_end;     // running total of the layers' block counts
        int vec;           // 16-byte path
    } layer[GCADA_MAX_WIDTHS - 1];
    int n_layers;
    const double* nring;
    const int32_t* tau;
    const uint8_t* hot;
    uint8_t* store_now;
};

template <typename T>
__global__ __launch_bounds__(256) void mlp_refresh_kernel(Hyper hy, RefreshArgs a)
{
    const int b = blockIdx.x;
    if (b >= a.layer[a.n_layers - 1].block_end) {
        if (a.store_now && threadIdx.x < kWave) store_flags_wave(hy, a.nring, a.tau, a.hot, a.store_now);
        return;
    }
    int li = 0;
    while (li + 1 < a.n_layers && b >= a.layer[li].block_end) ++li;
    const RefreshArgs::LayerCopy& y = a.layer[li];
    const int t = b - (li ? a.layer[li - 1].block_end : 0);
    const int bx = t % y.nbx, by = t / y.nbx;
    if (y.vec) weight_copy_block_vec<T>(bx, by, y.W, y.n_out, y.n_in, y.ld_in, y.ld_out, (T*)y.Wc, (T*)y.WcT);
    else weight_copy_block<T>(bx, by, y.W, y.n_out, y.n_in, y.ld_in, y.ld_out, (T*)y.Wc, (T*)y.WcT);
}

// Bias gradient of a layer from the transposed signal dZT [n][ldmu]: db[n] = sum_i dZ[i][n].
// The stale iterate's transposed signal is stored negated, so fresh - stale is a plain sum.
// All layers go into ONE launch (each is a few microseconds of work, less than a launch costs):
// grid: (sum over the layers of ceil(n_l/8), G), block 256: half a wave per hidden unit, both
// iterates, 16-byte loads (rows of dZT are padded to a multiple of 64 elements with zeros).
struct BiasArgs {
    struct LayerBias {
        const void* dZT;
        int64_t zt_it, zt_g;   // elements between the iterates / the groups
        int64_t boff;          // offset of the layer's biases in the parameter vector
        int nl, stat_off;
        int block_end;         // running total of the layers' block counts
    } layer[GCADA_MAX_WIDTHS - 1];
    int n_layers, ldmu;
    float* gbuf;
    const int32_t* which;
    double* part_stat;
    int n_stat;
};

// block `bi` of the launch's bias blocks, group g
template <typename T>
__device__ __forceinline__ void bias_grad_block(const Hyper& hy, const BiasArgs& b, int bi, int g)
{
    constexpr int V = 16 / (int)sizeof(T);
    __shared__ double s_red[4];
    int li = 0;
    while (li + 1 < b.n_layers && bi >= b.layer[li].block_end) ++li;
    const BiasArgs::LayerBias& y = b.layer[li];
    const int bx = bi - (li ? b.layer[li - 1].block_end : 0);
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int hl = lane & 31;                         // lane within the half wave
    const int n = bx * 8 + wave * 2 + (lane >> 5);
    double sq = 0;
    float s[2] = {0.0f, 0.0f};
    if (n < y.nl) {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const T* z = (const T*)y.dZT + (int64_t)it * y.zt_it + (int64_t)g * y.zt_g + (int64_t)n * b.ldmu;
            for (int i = hl * V; i < b.ldmu; i += 32 * V) {
                alignas(16) T v[V];
                *(uint4*)v = *(const uint4*)(z + i);
#pragma unroll
                for (int q = 0; q < V; ++q) s[it] += to_f<T>(v[q]);
            }
        }
    }
#pragma unroll
    for (int it = 0; it < 2; ++it)
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) s[it] += __shfl_xor(s[it], o, kWave);
    if (n < y.nl && hl == 0) {
        fresh_row(b.gbuf, b.which, hy, g)[y.boff + n] = s[0];
        const float df = s[0] + s[1];
        sq = (double)df * (double)df;
    }
    sq += __shfl_xor(sq, 32, kWave);
    if (lane == 0) s_red[wave] = sq;
    __syncthreads();
    if (threadIdx.x == 0)
        b.part_stat[(int64_t)g * b.n_stat + y.stat_off + bx] = s_red[0] + s_red[1] + s_red[2] + s_red[3];
}

template <typename T>
__global__ __launch_bounds__(256) void mlp_bias_grad(Hyper hy, BiasArgs b)
{
    const int g = blockIdx.y;
    if (hy.sel && !hy.sel[g]) return;            // unselected group (server-side rule)
    bias_grad_block<T>(hy, b, blockIdx.x, g);
}


// ---------------------------------------------------------------------------------------
// Weight gradient of a layer with few outputs (the output layer: M = n_l <= 16 classes) in fp32.
// In the general GEMM this product is a chain: every wave's accumulators take mu/2 dependent
// MFMA 32x32x2 per iterate whatever the tile, 22 of the 32 rows of a block are padding, and only
// a few dozen workgroups exist.  Here the 16 x 16 x 4 matrix instruction fits the shape (16 rows
// = the classes, 4 samples per instruction), and both operands are read row-major as they are (a
// lane loads element [sample s + lane/16][lane%16] of the signal and of the activations: 4 x 64
// contiguous bytes per operand and instruction).  A workgroup owns 16 columns of one group; each
// of its 16 waves takes a sixteenth of the samples, both iterates' loads in flight together; the
// waves' sums meet in LDS and are added in a fixed order.  Results as from the GEMM: fresh block
// -> gbuf, ||fresh - stale||^2 -> the partial slot of the column block (one per 16 columns).
constexpr int kNarrowCols = 16, kNarrowWaves = 16;
typedef float f32x4v __attribute__((ext_vector_type(4)));
struct DwNarrowArgs {
    Hyper hy;
    const float* A; int64_t a_it, a_g; int lda;    // activations of layer l-1 [mu][lda], per (iterate, group)
    const float* Z; int64_t z_it, z_g; int ldz;    // signal of layer l [mu][ldz] (not negated), pads zero
    int M, N, mu;
    float* gbuf; const int32_t* which; int64_t goff;
    double* part_stat; int n_stat, stat_off;
    const uint8_t* store_now;
};

// grid (ceil(N / 16), G), 1024 threads.  Accumulator register r of a lane is class
// 4 (lane / 16) + r, column lane % 16 of the block.
__global__ __launch_bounds__(kNarrowWaves * kWave) void mlp_dw_narrow(DwNarrowArgs a)
{
    __shared__ f32x4v s_part[2][kNarrowWaves][kWave];
    const Hyper& hy = a.hy;
    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int g = blockIdx.y, c0 = blockIdx.x * kNarrowCols;
    if (hy.sel && !hy.sel[g]) return;            // server-side rule / selected groups only
    const bool both = hy.sel == nullptr;         // otherwise: the gradient at theta^k, stored, nothing else
    const int per = ((a.mu + kNarrowWaves - 1) / kNarrowWaves + 3) / 4 * 4;
    const int s0 = min(a.mu, wave * per), s1 = min(a.mu, s0 + per);
    const int ks = lane >> 4, j = lane & 15, c = c0 + j;
    const bool c_ok = c < a.N;
    const float* Af = a.A + (int64_t)g * a.a_g;
    const float* Zf = a.Z + (int64_t)g * a.z_g;
    const float* As = Af + a.a_it;
    const float* Zs = Zf + a.z_it;
    f32x4v accf = {0, 0, 0, 0}, accs = {0, 0, 0, 0};
    constexpr int U = 8;                         // instructions per iterate whose operands are in flight together
    for (int s = s0; s < s1; s += 4 * U) {
        float zf[U], af[U], zs[U], as[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int ss = s + 4 * u + ks;
            const bool ok = ss < s1;
            zf[u] = ok ? global_load(Zf + (int64_t)ss * a.ldz + j) : 0.0f;
            af[u] = ok && c_ok ? global_load(Af + (int64_t)ss * a.lda + c) : 0.0f;
            zs[u] = ok && both ? global_load(Zs + (int64_t)ss * a.ldz + j) : 0.0f;
            as[u] = ok && both && c_ok ? global_load(As + (int64_t)ss * a.lda + c) : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            accf = __builtin_amdgcn_mfma_f32_16x16x4f32(zf[u], af[u], accf, 0, 0, 0);
            accs = __builtin_amdgcn_mfma_f32_16x16x4f32(zs[u], as[u], accs, 0, 0, 0);
        }
    }
    s_part[0][wave][lane] = accf;
    s_part[1][wave][lane] = accs;
    __syncthreads();
    if (wave != 0) return;
    f32x4v fresh = s_part[0][0][lane], stale = s_part[1][0][lane];
#pragma unroll
    for (int w = 1; w < kNarrowWaves; ++w) {     // fixed order over the waves
        fresh += s_part[0][w][lane];
        stale += s_part[1][w][lane];
    }
    const bool store = !both || !a.store_now || a.store_now[g];
    float* gb = fresh_row(a.gbuf, a.which, hy, g) + a.goff;
    double sq = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int m = 4 * (lane >> 4) + r;
        if (m < a.M && c_ok) {
            if (store) gb[(int64_t)m * a.N + c] = fresh[r];
            const float df = fresh[r] - stale[r];
            sq += (double)df * (double)df;
        }
    }
    if (!both) return;
    sq = wave_sum(sq);
    if (lane == 0) a.part_stat[(int64_t)g * a.n_stat + a.stat_off + blockIdx.x] = sq;
}

// ---------------------------------------------------------------------------------------
// First-layer statistic through two Gram matrices (bf16 models with the lazy gradient store).
// Both iterates see the same minibatch X (mu x n0), so the difference of the first layer's
// weight gradients is dZ^T X with dZ = dZ_1(theta^k) - dZ_1(theta_stale) (mu x n1), and
//     || dZ^T X ||_F^2 = sum_{s,s'} (X X^T)[s][s'] (dZ dZ^T)[s][s'],
// two mu x mu matrices instead of two n1 x n0 ones: 2 mu^2 (n0 + n1) flops instead of
// 4 mu n0 n1 (six times fewer for 3072-1024 at mu = 256), and no gradient is formed for a group
// that does not upload (paper Eq. (9): the statistic only decides; Sec. IV: only uploads enter
// the aggregate).
// One kernel forms a tile of both matrices in two accumulator sets and reduces their elementwise
// product; nothing mu x mu travels through memory.  The sum is bilinear, so the contraction of
// X X^T may be split over several workgroups (each also forms the whole dZ dZ^T tile, the cheaper
// of the two) and their partial statistics simply add up.
constexpr int kGramSplit = 1;      // workgroups per tile (shares of the X X^T contraction; more were measured slower)

struct GramArgs {
    Hyper hy;
    int M;                         // rows: the minibatch size
    int KX, KZ;                    // contraction lengths in elements: n0 and n1
    const ShardDesc* shards; const int32_t* idx;     // X: the minibatch rows of the shard, in place
    const void* dZd; int64_t z_g; int ldz;           // dZ: dZd + g * z_g + row * ldz
    double* part_stat; int n_stat, stat_off, n_slots;   // one partial per tile and share; the
                                                         // layer's other slots are cleared
};

// eight waves of 32 x 64 (two per SIMD: with four, one wave per SIMD had nobody to hide its
// waits behind; 56 -> 49 us for 3072-1024 at mu = 256), 128-byte k-tiles (-> 46.5 us)
using GramTile = Tile<128, 128, 128, 4, 2, 2>;

// acc += rows[m0..] rows[n0..]^T over the k-tiles [k_lo, k_hi) of 32 elements; rows at base + off.
// The tile is small, so a k-tile is little MFMA work against a trip to memory: FOUR k-tiles are in
// flight in four register sets (two LDS stages).  Iteration kt requests tile kt+4 into the set
// tile kt came from, multiplies tile kt and moves tile kt+1 to the other stage.  The loop body
// has no branches (the compiler then knows how many loads are outstanding at every wait and
// waits for the oldest only): the k-range is padded to a multiple of four tiles with tiles that
// are cleared on their way to LDS (not when they are loaded: that would wait for the load).
__device__ __forceinline__ void gram_loop(const char* base, const int64_t (&poff)[GramTile::PCH],
                                          const int64_t (&qoff)[GramTile::QCH], int k_lo, int k_hi, char* lds,
                                          f32x16 (&acc)[GramTile::TM][GramTile::TN])
{
    using TL = GramTile;
    constexpr int kP = TL::BM * TL::PITCH, NSET = 4;
    if (k_hi <= k_lo) return;                    // uniform
    const int last = k_hi - 1;
    u32x4 rp[NSET][TL::PCH], rq[NSET][TL::QCH];
    auto gload = [&](int kt, u32x4 (&p)[TL::PCH], u32x4 (&q)[TL::QCH]) {
        kt = kt <= last ? kt : last;
#pragma unroll
        for (int i = 0; i < TL::PCH; ++i) p[i] = global_load_vec(base + poff[i] + (int64_t)kt * TL::KROW);
#pragma unroll
        for (int i = 0; i < TL::QCH; ++i) q[i] = global_load_vec(base + qoff[i] + (int64_t)kt * TL::KROW);
    };
    auto clear_if_past = [&](int kt, u32x4 (&p)[TL::PCH], u32x4 (&q)[TL::QCH]) {
        const bool live = kt <= last;
#pragma unroll
        for (int i = 0; i < TL::PCH; ++i) p[i] = live ? p[i] : u32x4{0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < TL::QCH; ++i) q[i] = live ? q[i] : u32x4{0, 0, 0, 0};
    };
#pragma unroll
    for (int t = 0; t < NSET; ++t) gload(k_lo + t, rp[t], rq[t]);
    tile_lstore<TL>(lds, lds + kP, rp[0], rq[0]);
    __syncthreads();
    for (int kt0 = k_lo; kt0 < k_hi; kt0 += NSET) {
#pragma unroll
        for (int t = 0; t < NSET; ++t) {
            char* cur = lds + (t & 1) * TL::STAGE;
            char* nxt = lds + ((t + 1) & 1) * TL::STAGE;
            gload(kt0 + t + NSET, rp[t], rq[t]);
            tile_mma<bf16_t, TL>(cur, cur + kP, acc);
            clear_if_past(kt0 + t + 1, rp[(t + 1) % NSET], rq[(t + 1) % NSET]);
            tile_lstore<TL>(nxt, nxt + kP, rp[(t + 1) % NSET], rq[(t + 1) % NSET]);
            __syncthreads();
        }
    }
}

// grid: (ceil(M/128), ceil(M/128), G * kGramSplit).  Both matrices are symmetric: tiles below the
// diagonal do nothing, tiles above it count twice.
__global__ __launch_bounds__(GramTile::NT) void mlp_gram(GramArgs a)
{
    using TL = GramTile;
    extern __shared__ __align__(16) char lds[];
    constexpr int esz = 2;
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int wm = wave / TL::WN, wn = wave % TL::WN;
    // Workgroup -> (tile, group, share).  Consecutive workgroup ids go to different XCDs (id mod
    // 8), each with its own L2: the ids of one XCD are mapped to a contiguous range of work, so
    // that the tiles of one (group, share) -- which read the same rows -- meet in one L2.
    int bx, by, bz;
    {
        const int gx = gridDim.x, gy = gridDim.y, total = gx * gy * gridDim.z;
        int lin = blockIdx.x + gx * (blockIdx.y + gy * blockIdx.z);
        if (total % 8 == 0) lin = (lin % 8) * (total / 8) + lin / 8;
        bx = lin % gx; lin /= gx;
        by = lin % gy;
        bz = lin / gy;
    }
    const int g = bz / kGramSplit, sp = bz % kGramSplit;
    const int tile = by * gridDim.x + bx, ntile = gridDim.x * gridDim.y;
    double* out = a.part_stat + (int64_t)g * a.n_stat + a.stat_off;
    if (bx < by) {
        if (tid == 0) out[tile * kGramSplit + sp] = 0.0;
        return;
    }
    const int m0 = by * TL::BM, n0 = bx * TL::BN;
    f32x16 accx[TL::TM][TL::TN], accz[TL::TM][TL::TN];
#pragma unroll
    for (int i = 0; i < TL::TM; ++i)
#pragma unroll
        for (int j = 0; j < TL::TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) { accx[i][j][e] = 0.0f; accz[i][j][e] = 0.0f; }
    constexpr int kElems = TL::KROW / esz;
    int64_t poff[TL::PCH], qoff[TL::QCH];
    {
        // X X^T, this share of the contraction: the minibatch rows of the shard (rows past M: row 0
        // of the minibatch, result unused)
        const ShardDesc sh = a.shards[g];
        auto row_off = [&](int m) -> int64_t {
            if (m >= a.M) m = 0;
            int64_t row;
            if (a.idx) row = a.idx[(int64_t)g * a.hy.mu + m];
            else row = (int64_t)(((unsigned long long)a.hy.k * (unsigned long long)a.hy.mu +
                                  (unsigned long long)m) % (unsigned long long)sh.rows);
            return row * sh.ld * esz;
        };
#pragma unroll
        for (int i = 0; i < TL::PCH; ++i)
            poff[i] = row_off(m0 + (tid + TL::NT * i) / TL::CPR) + ((tid + TL::NT * i) % TL::CPR) * 16;
#pragma unroll
        for (int i = 0; i < TL::QCH; ++i)
            qoff[i] = row_off(n0 + (tid + TL::NT * i) / TL::CPR) + ((tid + TL::NT * i) % TL::CPR) * 16;
        const int nk = (a.KX + kElems - 1) / kElems;
        gram_loop((const char*)sh.X, poff, qoff, (int)((int64_t)nk * sp / kGramSplit),
                  (int)((int64_t)nk * (sp + 1) / kGramSplit), lds, accx);
    }
    {
        // dZ dZ^T, whole
        auto row_off = [&](int m) -> int64_t { return (int64_t)(m < a.M ? m : 0) * a.ldz * esz; };
#pragma unroll
        for (int i = 0; i < TL::PCH; ++i)
            poff[i] = row_off(m0 + (tid + TL::NT * i) / TL::CPR) + ((tid + TL::NT * i) % TL::CPR) * 16;
#pragma unroll
        for (int i = 0; i < TL::QCH; ++i)
            qoff[i] = row_off(n0 + (tid + TL::NT * i) / TL::CPR) + ((tid + TL::NT * i) % TL::CPR) * 16;
        const int nk = (a.KZ + kElems - 1) / kElems;
        gram_loop((const char*)a.dZd + (int64_t)g * a.z_g * esz, poff, qoff, 0, nk, lds, accz);
    }
    // accumulator element e of a lane: column n = lane % 32, row m = (e/4)*8 + (lane/32)*4 + e%4
    constexpr int RW = TL::BM / TL::WM, CW = TL::BN / TL::WN;
    const int cl = lane & 31, rh = (lane >> 5) * 4;
    double sq = 0;
#pragma unroll
    for (int i = 0; i < TL::TM; ++i)
#pragma unroll
        for (int j = 0; j < TL::TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + wm * RW + i * 32 + (e >> 2) * 8 + rh + (e & 3);
                const int n = n0 + wn * CW + j * 32 + cl;
                if (m < a.M && n < a.M) sq += (double)accx[i][j][e] * (double)accz[i][j][e];
            }
    if (bx > by) sq *= 2.0;                       // the mirrored tile below the diagonal
    sq = wave_sum(sq);
    double* red = (double*)lds;                   // every wave is past the last barrier of the k loops
    if (lane == 0) red[wave] = sq;
    __syncthreads();
    if (tid == 0) {
        double t = 0;
#pragma unroll
        for (int wv = 0; wv < TL::NW; ++wv) t += red[wv];
        out[tile * kGramSplit + sp] = t;
    }
    // the layer's remaining slots belong to the weight-gradient tiles of the other method
    if (tile == 0 && sp == 0)
        for (int q = ntile * kGramSplit + tid; q < a.n_slots; q += TL::NT) out[q] = 0.0;
}

// dZd[g][s][n] = dZ[0][g][s][n] - dZ[1][g][s][n] (the signal of the fresh minus that of the stale
// iterate), and -- the same read -- the first layer's bias gradient: its fresh value
// sum_s dZ[0][g][s][n] goes to the group's fresh row, the squared difference of the two iterates'
// sums into the layer's bias slots of the statistic.  The workgroups past the first ld / 64 form
// the bias gradients of the deeper layers (one launch less).
// grid: (ld / 64 + bias blocks of `deeper`, G), block 256 = 8 column chunks of 8 x 32 row lanes;
// ld a multiple of 64.
__global__ __launch_bounds__(256) void mlp_signal_diff_bias(Hyper hy, int n1, int ld, const bf16_t* __restrict__ z0,
                                                            const bf16_t* __restrict__ z1, bf16_t* __restrict__ out,
                                                            float* __restrict__ gbuf, const int32_t* __restrict__ which,
                                                            int64_t boff, double* __restrict__ part_stat, int n_stat,
                                                            int stat_off, int n_slots, BiasArgs deeper)
{
    const int n_cb = ld / 64;
    if ((int)blockIdx.x >= n_cb) {
        bias_grad_block<bf16_t>(hy, deeper, (int)blockIdx.x - n_cb, blockIdx.y);
        return;
    }
    __shared__ float s_f[32][64 + 1], s_d[32][64 + 1];
    const int g = blockIdx.y, cb = blockIdx.x;
    const int chunk = threadIdx.x % 8, rl = threadIdx.x / 8;
    const int64_t base = (int64_t)g * hy.mu * ld + cb * 64 + chunk * 8;
    float fs[8], ds[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) fs[e] = ds[e] = 0.0f;
    for (int r = rl; r < hy.mu; r += 32) {
        alignas(16) bf16_t p[8], q[8], d[8];
        *(uint4*)p = *(const uint4*)(z0 + base + (int64_t)r * ld);
        *(uint4*)q = *(const uint4*)(z1 + base + (int64_t)r * ld);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float a = to_f<bf16_t>(p[e]);
            d[e] = to_T<bf16_t>(a - to_f<bf16_t>(q[e]));
            fs[e] += a;
            // the difference of the bias gradients sums the two signals themselves (what the
            // weight-gradient route adds up too), not the rounded difference
            ds[e] += a - to_f<bf16_t>(q[e]);
        }
        *(uint4*)(out + base + (int64_t)r * ld) = *(const uint4*)d;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) { s_f[rl][chunk * 8 + e] = fs[e]; s_d[rl][chunk * 8 + e] = ds[e]; }
    __syncthreads();
    double sq = 0;
    if (threadIdx.x < 64) {
        float f = 0.0f, d = 0.0f;
        for (int r = 0; r < 32; ++r) { f += s_f[r][threadIdx.x]; d += s_d[r][threadIdx.x]; }   // fixed order
        const int n = cb * 64 + threadIdx.x;
        if (n < n1) {
            fresh_row(gbuf, which, hy, g)[boff + n] = f;
            sq = (double)d * (double)d;
        }
    }
    if (threadIdx.x < kWave) {
        sq = wave_sum(sq);
        double* slots = part_stat + (int64_t)g * n_stat + stat_off;
        if (threadIdx.x == 0) slots[cb] = sq;
        // the layer's remaining bias slots belong to the blocks of the other method
        if (cb == 0)
            for (int q = n_cb + threadIdx.x; q < n_slots; q += kWave) slots[q] = 0.0;
    }
}

}  // namespace

// ---------------------------------------------------------------------------------------
struct MlpWork {
    Layout lay{};
    bool bf16 = false;
    int esz = 4;
    // per layer l (index l): activations A_l, AT_l (l = 1..L-1), signals dZ_l, dZT_l (l = 1..L)
    void* Xg = nullptr; void* XgT = nullptr;
    void* A[GCADA_MAX_WIDTHS] = {};  void* AT[GCADA_MAX_WIDTHS] = {};
    void* dZ[GCADA_MAX_WIDTHS] = {}; void* dZT[GCADA_MAX_WIDTHS] = {};
    void* relu[GCADA_MAX_WIDTHS] = {};   // l = 1..L-1: one bit per element of A_l (see GemmArgs::relu_bits)
    // weight copies per ring slot: Wc_l [slot][n_l][ld_{l-1}], WcT_l [slot][n_{l-1}][ld_l]
    void* Wc[GCADA_MAX_WIDTHS] = {}; void* WcT[GCADA_MAX_WIDTHS] = {};
    int64_t wc_slot[GCADA_MAX_WIDTHS] = {}, wct_slot[GCADA_MAX_WIDTHS] = {};
    // partial-statistic slots
    int stat_off_w[GCADA_MAX_WIDTHS] = {}, stat_off_b[GCADA_MAX_WIDTHS] = {};
    int n_stat = 0, n_loss = 0;
    bool small = false;              // 64 x 64 GEMM tiles (small fp32 problems)
    int n_cu = 1;                    // compute units of the device
    // first-layer statistic through Gram matrices (see mlp_gram)
    bool gram_ok = false;            // shapes and type allow it and it is the cheaper way
    bool gram_active = false;        // the last gradient stage used it
    const int32_t* idx_last = nullptr;   // that stage's minibatch ids (for the second gather)
    void* dZd = nullptr;             // T [G][mu][ld_1]
    size_t slack = 0;
    std::vector<void*> allocs;
};

static hipError_t walloc(MlpWork* w, void** p, size_t bytes)
{
    // slack: GEMM tiles read whole tiles of rows, also past the end of the last batch entry
    bytes += w->slack;
    hipError_t e = hipMalloc(p, bytes);
    if (e != hipSuccess) return e;
    w->allocs.push_back(*p);
    return hipMemset(*p, 0, bytes);
}

hipError_t mlp_plan(gcada_ctx* c)
{
    auto* w = new MlpWork();
    c->mlp = w;
    const gcada_dims& d = c->dims;
    Layout& lay = w->lay;
    lay.L = d.n_widths - 1;
    w->bf16 = d.dtype == GCADA_BF16;
    w->esz = w->bf16 ? 2 : 4;
    int64_t off = 0;
    for (int l = 0; l <= lay.L; ++l) {
        lay.n[l] = d.widths[l];
        lay.ld[l] = round_up(d.widths[l], 64);
        if (l >= 1) {
            lay.woff[l] = off;
            off += (int64_t)lay.n[l] * lay.n[l - 1];
            lay.boff[l] = off;
            off += lay.n[l];
        }
    }
    if (lay.n[lay.L] > kHeadClasses) return hipErrorInvalidValue;
    const int mu = c->hy.mu, G = c->hy.G, L = lay.L, nslot = c->hy.D + 1;
    lay.ldmu = round_up(mu, 64);
    int maxld = lay.ldmu;
    for (int l = 0; l <= L; ++l) maxld = std::max(maxld, lay.ld[l]);
    w->slack = (size_t)256 * maxld * 4 + 256;      // a tile may read up to 256 rows past an operand's end
    const size_t es = w->esz;
    hipError_t e;
    if ((e = walloc(w, &w->Xg, (size_t)G * mu * lay.ld[0] * es)) != hipSuccess) return e;
    if ((e = walloc(w, &w->XgT, (size_t)G * lay.n[0] * lay.ldmu * es)) != hipSuccess) return e;
    for (int l = 1; l <= L; ++l) {
        const size_t rm = (size_t)2 * G * mu * lay.ld[l] * es, tr = (size_t)2 * G * lay.n[l] * lay.ldmu * es;
        if (l < L) {
            if ((e = walloc(w, &w->A[l], rm)) != hipSuccess) return e;
            if ((e = walloc(w, &w->AT[l], tr)) != hipSuccess) return e;
            // whole tiles of at most 256 x 256, 16 elements per 2-byte word
            const size_t bits = (size_t)2 * G * (mu + 256) * (lay.n[l] + 256) / 16 * 2;
            if ((e = walloc(w, &w->relu[l], bits)) != hipSuccess) return e;
        }
        if ((e = walloc(w, &w->dZ[l], rm)) != hipSuccess) return e;
        if ((e = walloc(w, &w->dZT[l], tr)) != hipSuccess) return e;
        w->wc_slot[l] = (int64_t)lay.n[l] * lay.ld[l - 1];
        w->wct_slot[l] = (int64_t)lay.n[l - 1] * lay.ld[l];
        if ((e = walloc(w, &w->Wc[l], (size_t)nslot * w->wc_slot[l] * es)) != hipSuccess) return e;
        if (l > 1 && (e = walloc(w, &w->WcT[l], (size_t)nslot * w->wct_slot[l] * es)) != hipSuccess) return e;
    }
    // small tiles when the first forward GEMM in 128 x 128 tiles cannot give every compute unit
    // two workgroups
    {
        hipDeviceProp_t prop;
        if ((e = hipGetDeviceProperties(&prop, c->device)) != hipSuccess) return e;
        const int64_t wgs = (int64_t)((mu + 127) / 128) * ((lay.n[1] + 127) / 128) * 2 * G;
        w->small = !w->bf16 && wgs < 2 * (int64_t)prop.multiProcessorCount;
        w->n_cu = prop.multiProcessorCount;
    }
    // partial statistics: per layer the weight-gradient tiles and the bias blocks
    int ns = 0;
    for (int l = 1; l <= L; ++l) {
        w->stat_off_w[l] = ns;
        if (dw_narrow_layer(w->bf16, w->small, l, lay.n[l])) ns += (lay.n[l - 1] + 15) / 16;
        else ns += w->bf16 ? dw_blocks<bf16_t>(lay.n[l], lay.n[l - 1], w->small)
                           : dw_blocks<float>(lay.n[l], lay.n[l - 1], w->small);
        w->stat_off_b[l] = ns;
        ns += (lay.n[l] + 7) / 8;
    }
    w->n_stat = ns;
    // Gram statistic of the first layer: bf16 only (the statistic's tolerance there absorbs the
    // rounding of the signal difference), when it needs at most half the flops of the two
    // weight-gradient passes, and its tiles fit the layer's partial slots
    {
        const int64_t n0 = lay.n[0], n1 = lay.n[1];
        const int gt = (mu + GramTile::BM - 1) / GramTile::BM;
        if (w->bf16 && (int64_t)mu * (n0 + n1) <= n0 * n1 &&
            gt * gt * kGramSplit <= dw_blocks<bf16_t>(lay.n[1], lay.n[0], false)) {
            if ((e = walloc(w, &w->dZd, (size_t)G * mu * lay.ld[1] * es)) != hipSuccess) return e;
            constexpr int glds = 2 * GramTile::STAGE;
            if ((e = hipFuncSetAttribute((const void*)mlp_gram, hipFuncAttributeMaxDynamicSharedMemorySize, glds)) != hipSuccess) return e;
            w->gram_ok = true;
        }
    }
    w->n_loss = w->bf16 ? head_row_blocks<bf16_t>(mu, w->small, lay.n[lay.L])
                        : head_row_blocks<float>(mu, w->small, lay.n[lay.L]);
    c->n_stat_part = std::max(c->n_stat_part, ns);
    c->n_loss_part = std::max(c->n_loss_part, w->n_loss);
    return hipSuccess;
}

void mlp_free(gcada_ctx* c)
{
    if (!c->mlp) return;
    for (void* p : c->mlp->allocs) (void)hipFree(p);
    delete c->mlp;
    c->mlp = nullptr;
}

template <typename T>
static hipError_t refresh_slot_t(gcada_ctx* c, int slot, bool flags, hipStream_t s)
{
    MlpWork* w = c->mlp;
    const Layout& lay = w->lay;
    const float* th = c->ring + (int64_t)slot * c->hy.pstride;
    RefreshArgs a{};
    int blocks = 0;
    for (int l = 1; l <= lay.L; ++l) {
        RefreshArgs::LayerCopy& y = a.layer[l - 1];
        y.W = th + lay.woff[l];
        y.Wc = (T*)w->Wc[l] + (int64_t)slot * w->wc_slot[l];
        // the transpose serves the signal of layer l-1, which the first layer does not need
        y.WcT = l > 1 ? (T*)w->WcT[l] + (int64_t)slot * w->wct_slot[l] : nullptr;
        y.n_out = lay.n[l]; y.n_in = lay.n[l - 1]; y.ld_in = lay.ld[l - 1]; y.ld_out = lay.ld[l];
        y.nbx = (lay.n[l - 1] + 63) / 64;
        blocks += y.nbx * ((lay.n[l] + 63) / 64);
        y.block_end = blocks;
        y.vec = lay.n[l - 1] % 4 == 0 && lay.woff[l] % 4 == 0;
    }
    a.n_layers = lay.L;
    if (flags) { a.nring = c->nring; a.tau = c->tau; a.hot = c->hot; a.store_now = c->store_now; }
    mlp_refresh_kernel<T><<<blocks + 1, 256, 0, s>>>(c->hy, a);
    return hipGetLastError();
}

hipError_t mlp_refresh_slot(gcada_ctx* c, int slot, bool flags, hipStream_t s)
{
    return c->mlp->bf16 ? refresh_slot_t<bf16_t>(c, slot, flags, s) : refresh_slot_t<float>(c, slot, flags, s);
}

hipError_t mlp_refresh_weights(gcada_ctx* c, hipStream_t s)
{
    for (int slot = 0; slot <= c->hy.D; ++slot) {
        hipError_t e = mlp_refresh_slot(c, slot, false, s);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Weight-gradient GEMM of layer l.  hy.sel == nullptr: both iterates, the statistic, and the
// fresh block of the groups with store_now[g] (all groups when store_now is null).  hy.sel given:
// the gradient at theta^k of the groups with sel[g], stored; nothing else.
static GemmArgs dw_args(gcada_ctx* c, int l, const Hyper& hy, const uint8_t* store_now)
{
    MlpWork* w = c->mlp;
    const Layout& lay = w->lay;
    const int G = hy.G;
    GemmArgs a{};
    a.hy = hy; a.tau = c->tau; a.G = G;
    a.M = lay.n[l]; a.N = lay.n[l - 1]; a.K = hy.mu;
    a.P = w->dZT[l]; a.p_it = (int64_t)G * lay.n[l] * lay.ldmu; a.p_g = (int64_t)lay.n[l] * lay.ldmu;
    a.ldp = lay.ldmu;
    if (l == 1) { a.Q = w->XgT; a.q_it = 0; a.q_g = (int64_t)lay.n[0] * lay.ldmu; }
    else { a.Q = w->AT[l - 1]; a.q_it = (int64_t)G * lay.n[l - 1] * lay.ldmu; a.q_g = (int64_t)lay.n[l - 1] * lay.ldmu; }
    a.ldq = lay.ldmu; a.q_is_weight = 0;
    a.gbuf = c->gbuf; a.which = c->which; a.goff = lay.woff[l];
    a.part_stat = c->part_stat; a.n_stat = w->n_stat; a.stat_off = w->stat_off_w[l];
    a.store_now = store_now;
    return a;
}

template <typename T>
static bool dw_narrow_layer(const gcada_ctx* c, int l)
{
    return sizeof(T) == 4 && dw_narrow_layer(c->mlp->bf16, c->mlp->small, l, c->mlp->lay.n[l]);
}
static hipError_t launch_dw_narrow(gcada_ctx* c, int l, const Hyper& hy, const uint8_t* store_now, hipStream_t s)
{
    MlpWork* w = c->mlp;
    const Layout& lay = w->lay;
    const int G = hy.G, mu = hy.mu;
    DwNarrowArgs a{};
    a.hy = hy;
    a.A = (const float*)w->A[l - 1]; a.a_it = (int64_t)G * mu * lay.ld[l - 1]; a.a_g = (int64_t)mu * lay.ld[l - 1];
    a.lda = lay.ld[l - 1];
    a.Z = (const float*)w->dZ[l]; a.z_it = (int64_t)G * mu * lay.ld[l]; a.z_g = (int64_t)mu * lay.ld[l];
    a.ldz = lay.ld[l];
    a.M = lay.n[l]; a.N = lay.n[l - 1]; a.mu = mu;
    a.gbuf = c->gbuf; a.which = c->which; a.goff = lay.woff[l];
    a.part_stat = c->part_stat; a.n_stat = w->n_stat; a.stat_off = w->stat_off_w[l];
    a.store_now = store_now;
    mlp_dw_narrow<<<dim3((a.N + kNarrowCols - 1) / kNarrowCols, G), kNarrowWaves * kWave, 0, s>>>(a);
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_dw(gcada_ctx* c, int l, const Hyper& hy, const uint8_t* store_now, hipStream_t s)
{
    if (dw_narrow_layer<T>(c, l)) return launch_dw_narrow(c, l, hy, store_now, s);
    return launch_gemm<T, EPI_DW>(dw_args(c, l, hy, store_now), hy.G, c->mlp->small, s);
}

// all layers' weight gradients at theta^k of the groups in hy.sel, one launch
template <typename T, bool SMALL>
static hipError_t launch_dw_selected(gcada_ctx* c, const Hyper& hy, const uint8_t* first_layer_sel, hipStream_t s)
{
    using TL = typename TileOf<T, EPI_DW, SMALL>::type;
    const int lds = gemm_lds_bytes<T, EPI_DW, TL>() + 2 * hy.G * (int)sizeof(uint16_t);
    static int attr_lds = 0;
    if (lds > attr_lds) {
        hipError_t e = hipFuncSetAttribute((const void*)mlp_dw_selected<T, TL>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        attr_lds = lds;
    }
    const Layout& lay = c->mlp->lay;
    DwSelectedArgs a{};
    // (a layer that the gradient stage handles with the narrow kernel is recomputed by that kernel:
    // the same sums in the same order; such layers are the last ones)
    int top = lay.L;
    while (top >= 1 && dw_narrow_layer<T>(c, top)) {
        hipError_t e = launch_dw_narrow(c, top, hy, nullptr, s);
        if (e != hipSuccess) return e;
        --top;
    }
    a.n_layers = top;
    int tiles = 0;
    for (int l = 1; l <= top; ++l) {
        a.layer[l - 1] = dw_args(c, l, hy, nullptr);
        tiles += ((lay.n[l] + TL::BM - 1) / TL::BM) * ((lay.n[l - 1] + TL::BN - 1) / TL::BN);
        a.tile_end[l - 1] = tiles;
    }
    a.sel_rest = hy.sel;
    a.sel_first = first_layer_sel ? first_layer_sel : hy.sel;
    const int64_t most = (int64_t)tiles * hy.G;
    const int grid = (int)std::min<int64_t>(most, c->mlp->n_cu);
    mlp_dw_selected<T, TL><<<grid, TL::NT, lds, s>>>(a);
    return hipGetLastError();
}

// Arguments of the bias gradients of layers l_lo .. L (none: n_layers = 0).
static BiasArgs bias_args(gcada_ctx* c, int l_lo, int* blocks)
{
    MlpWork* w = c->mlp;
    const Layout& lay = w->lay;
    const int G = c->hy.G;
    BiasArgs b{};
    int total = 0;
    for (int l = l_lo; l <= lay.L; ++l) {
        BiasArgs::LayerBias& y = b.layer[b.n_layers++];
        y.dZT = w->dZT[l];
        y.zt_it = (int64_t)G * lay.n[l] * lay.ldmu;
        y.zt_g = (int64_t)lay.n[l] * lay.ldmu;
        y.boff = lay.boff[l];
        y.nl = lay.n[l];
        y.stat_off = w->stat_off_b[l];
        total += (lay.n[l] + 7) / 8;
        y.block_end = total;
    }
    b.ldmu = lay.ldmu;
    b.gbuf = c->gbuf; b.which = c->which; b.part_stat = c->part_stat; b.n_stat = w->n_stat;
    *blocks = total;
    return b;
}

// Statistic of the first layer's weights from the two Gram matrices (bf16): the signal
// difference, then one kernel that forms both matrices tile by tile and sums their product into
// the layer's partial slots.
static hipError_t gram_statistic(gcada_ctx* c, const int32_t* idx, hipStream_t s)
{
    MlpWork* w = c->mlp;
    const Layout& lay = w->lay;
    const int G = c->hy.G, mu = c->hy.mu;
    const int64_t count = (int64_t)G * mu * lay.ld[1];
    const bf16_t* z0 = (const bf16_t*)w->dZ[1];
    int bias_blocks = 0;
    const BiasArgs deeper = bias_args(c, 2, &bias_blocks);
    mlp_signal_diff_bias<<<dim3(lay.ld[1] / 64 + bias_blocks, G), 256, 0, s>>>(
        c->hy, lay.n[1], lay.ld[1], z0, z0 + count, (bf16_t*)w->dZd, c->gbuf, c->which, lay.boff[1], c->part_stat,
        w->n_stat, w->stat_off_b[1], (lay.n[1] + 7) / 8, deeper);
    constexpr int glds = 2 * GramTile::STAGE;
    const int gt = (mu + GramTile::BM - 1) / GramTile::BM;
    GramArgs a{};
    a.hy = c->hy; a.M = mu; a.KX = lay.n[0]; a.KZ = lay.n[1];
    a.shards = c->d_shards; a.idx = idx;
    a.dZd = w->dZd; a.z_g = (int64_t)mu * lay.ld[1]; a.ldz = lay.ld[1];
    a.part_stat = c->part_stat; a.n_stat = w->n_stat; a.stat_off = w->stat_off_w[1];
    a.n_slots = w->stat_off_b[1] - w->stat_off_w[1];
    mlp_gram<<<dim3(gt, gt, G * kGramSplit), GramTile::NT, glds, s>>>(a);
    return hipGetLastError();
}

template <typename T>
static hipError_t mlp_gradients_t(gcada_ctx* c, const int32_t* idx, hipStream_t s)
{
    MlpWork* w = c->mlp;
    const Layout& lay = w->lay;
    const Hyper& hy = c->hy;
    const int G = hy.G, mu = hy.mu, L = lay.L;
    hipError_t e;
    // 1. gather the minibatch rows: transposed always; row-major only when the first forward
    //    GEMM cannot read the shard rows in place (rows not 16-byte aligned, or a width whose
    //    last k-tile would reach past the end of a row)
    constexpr int V = 16 / (int)sizeof(T);
    bool vec_ok = lay.n[0] % V == 0;
    for (const auto& sd : c->shards)
        if ((sd.ld * (int64_t)sizeof(T)) % 16 || ((uintptr_t)sd.X % 16)) vec_ok = false;
    const bool in_place = vec_ok && (lay.n[0] * (int)sizeof(T)) % TileOf<T, EPI_FWD, false>::type::KROW == 0;
    // first-layer statistic through Gram matrices: then this stage forms no first-layer weight
    // gradient and needs no transposed minibatch
    const bool gram = w->gram_ok && c->allow_gram && c->lazy_store && !hy.sel && in_place;
    w->gram_active = gram;
    w->idx_last = idx;
    if (gram) {
        // nothing to gather: the forward GEMM and the Gram kernel read the rows in place, and the
        // transposed minibatch serves only the weight gradient, which follows the selection
    } else if (vec_ok) {
        dim3 grid((lay.n[0] + 8 * V - 1) / (8 * V), (mu + 63) / 64, G);
        mlp_gather_vec<T><<<grid, 256, 0, s>>>(hy, c->d_shards, idx, lay.n[0], lay.ld[0], lay.ldmu,
                                                in_place ? nullptr : (T*)w->Xg, (T*)w->XgT, DenseTranspose<T>{});
    } else {
        dim3 grid((lay.n[0] + 63) / 64, (mu + 63) / 64, G);
        mlp_gather<T><<<grid, 256, 0, s>>>(hy, c->d_shards, idx, lay.n[0], lay.ld[0], lay.ldmu,
                                            (T*)w->Xg, (T*)w->XgT);
    }
    auto rm_it = [&](int l) { return (int64_t)G * mu * lay.ld[l]; };       // iterate stride, row-major
    auto rm_g = [&](int l) { return (int64_t)mu * lay.ld[l]; };
    auto tr_it = [&](int l) { return (int64_t)G * lay.n[l] * lay.ldmu; };  // transposed
    auto tr_g = [&](int l) { return (int64_t)lay.n[l] * lay.ldmu; };
    // 2. forward: hidden layers (bias + ReLU), then the output layer with its loss
    for (int l = 1; l <= L; ++l) {
        GemmArgs a{};
        a.hy = hy; a.tau = c->tau; a.G = G;
        a.M = mu; a.N = lay.n[l]; a.K = lay.n[l - 1];
        if (l == 1 && in_place) { a.gather = 1; a.shards = c->d_shards; a.idx = idx; }
        else if (l == 1) { a.P = w->Xg; a.p_it = 0; a.p_g = rm_g(0); a.ldp = lay.ld[0]; }
        else { a.P = w->A[l - 1]; a.p_it = rm_it(l - 1); a.p_g = rm_g(l - 1); a.ldp = lay.ld[l - 1]; }
        a.Q = w->Wc[l]; a.q_is_weight = 1; a.q_slot = w->wc_slot[l]; a.ldq = lay.ld[l - 1];
        a.ring = c->ring; a.boff = lay.boff[l];
        if (l < L) {
            a.O = w->A[l]; a.o_it = rm_it(l); a.o_g = rm_g(l); a.ldo = lay.ld[l];
            a.OT = w->AT[l]; a.t_it = tr_it(l); a.t_g = tr_g(l); a.ldt = lay.ldmu;
            a.relu_bits = (uint16_t*)w->relu[l];
            if ((e = launch_gemm<T, EPI_FWD>(a, 2 * G, w->small, s)) != hipSuccess) return e;
        } else {
            a.O = w->dZ[L]; a.o_it = rm_it(L); a.o_g = rm_g(L); a.ldo = lay.ld[L];
            a.OT = w->dZT[L]; a.t_it = tr_it(L); a.t_g = tr_g(L); a.ldt = lay.ldmu;
            a.shards = c->d_shards; a.idx = idx; a.part_loss = c->part_loss;
            if ((e = launch_gemm<T, EPI_HEAD>(a, 2 * G, w->small, s)) != hipSuccess) return e;
        }
    }
    // 3. backward, layer by layer
    for (int l = L; l >= 1; --l) {
        if (l == 1 && gram) {
            // (the gradient itself is formed after the selection, for the groups that upload)
            if ((e = gram_statistic(c, idx, s)) != hipSuccess) return e;
        } else {
            // weight gradient of layer l, both iterates in one workgroup
            if ((e = launch_dw<T>(c, l, hy, c->lazy_store && !hy.sel ? c->store_now : nullptr, s)) != hipSuccess)
                return e;
        }
        if (l > 1) {   // signal of layer l-1: dZ_{l-1} = (dZ_l W_l) * [a_{l-1} > 0]
            GemmArgs a{};
            a.hy = hy; a.tau = c->tau; a.G = G;
            a.M = mu; a.N = lay.n[l - 1]; a.K = lay.n[l];
            a.P = w->dZ[l]; a.p_it = rm_it(l); a.p_g = rm_g(l); a.ldp = lay.ld[l];
            a.Q = w->WcT[l]; a.q_is_weight = 1; a.q_slot = w->wct_slot[l]; a.ldq = lay.ld[l];
            a.relu_bits = (uint16_t*)w->relu[l - 1];
            a.O = w->dZ[l - 1]; a.o_it = rm_it(l - 1); a.o_g = rm_g(l - 1); a.ldo = lay.ld[l - 1];
            a.OT = w->dZT[l - 1]; a.t_it = tr_it(l - 1); a.t_g = tr_g(l - 1); a.ldt = lay.ldmu;
            // with the Gram statistic the transposed first-layer signal serves only the weight
            // gradient of uploading groups
            if (l - 1 == 1 && gram) a.t_flags = c->store_now;
            if ((e = launch_gemm<T, EPI_DA>(a, 2 * G, w->small, s)) != hipSuccess) return e;
        }
    }
    // bias gradients of all layers in one launch (with the Gram statistic the signal-difference
    // launch has formed them)
    if (!gram) {
        int bias_blocks = 0;
        const BiasArgs b = bias_args(c, 1, &bias_blocks);
        mlp_bias_grad<T><<<dim3(bias_blocks, G), 256, 0, s>>>(hy, b);
    }
    c->n_stat_used = w->n_stat;
    c->n_loss_used = G * w->n_loss;
    return hipGetLastError();
}

// whether the last gradient stage took the first layer's statistic from the Gram matrices
bool mlp_gram_active(const gcada_ctx* c) { return c->mlp && c->mlp->gram_active; }

hipError_t mlp_gradients(gcada_ctx* c, const int32_t* idx, hipStream_t s)
{
    return c->mlp->bf16 ? mlp_gradients_t<bf16_t>(c, idx, s) : mlp_gradients_t<float>(c, idx, s);
}

// Second half of the lazy gradient store: the weight gradients at theta^k of the groups in
// c->redo (selected, but not written by the gradient stage) are recomputed from the signals and
// activations the stage left behind -- the same k-tiles in the same order, so the same bits --
// and written to their fresh rows.
hipError_t mlp_store_selected(gcada_ctx* c, hipStream_t s)
{
    Hyper hy = c->hy;
    hy.sel = c->redo;
    const uint8_t* first = nullptr;
    if (c->mlp->gram_active) {
        // With the Gram statistic the gradient stage has formed no first-layer weight gradient at
        // all: every selected group gets it here, from its transposed minibatch, which is
        // gathered now (bf16, 16-byte rows: see the conditions of the Gram statistic).
        first = c->mask;
        Hyper hg = c->hy;
        hg.sel = first;
        // The same launch transposes the first-layer signal of the groups that are selected
        // without having been flagged: the gradient stage wrote the transposed copy only for
        // the flagged ones.
        const Layout& lay = c->mlp->lay;
        DenseTranspose<bf16_t> dt{(const bf16_t*)c->mlp->dZ[1], (bf16_t*)c->mlp->dZT[1], lay.n[1], lay.ld[1], c->redo};
        dim3 grid((lay.n[0] + 63) / 64 + (lay.n[1] + 63) / 64, (hy.mu + 63) / 64, hy.G);
        mlp_gather_vec<bf16_t><<<grid, 256, 0, s>>>(hg, c->d_shards, c->mlp->idx_last, lay.n[0], lay.ld[0],
                                                     lay.ldmu, nullptr, (bf16_t*)c->mlp->XgT, dt);
    }
    if (c->mlp->bf16) return launch_dw_selected<bf16_t, false>(c, hy, first, s);
    return c->mlp->small ? launch_dw_selected<float, true>(c, hy, first, s)
                         : launch_dw_selected<float, false>(c, hy, first, s);
}

}  // namespace gcada
