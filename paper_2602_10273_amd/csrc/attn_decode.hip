// Single-token decode attention that reads the particle caches where the reorder step (Alg. 1 "reorder KV cache by
// A"; App. C) leaves them: the double-buffered rows (row r lives in buffer parity[r]) or the paged pools (through the
// page table).  Not part of the paper's method: it is the consumer a decoder needs so that neither layout has to be
// repacked before attention.  Textbook scaled dot-product attention with grouped query heads:
//     s_j = scale <q[r, h G + g], K[r, h, j]>,  p = softmax_j s,  out[r, h G + g] = sum_j p_j V[r, h, j],  j < len.
//
// gfx950 design.  The kernel is a stream over K and V (each read once, 16-byte loads); the two contractions run on the
// matrix cores so that the vector ALUs only see the softmax.  One workgroup of 2 waves per (row, KV head, split of the
// positions); a wave walks tiles of 16 positions:
//   scores   S^T[pos, head] = K_tile[pos, dim] Q^T[dim, head]: 16x16x16 bf16 MFMA, A = the K tile exactly as loaded
//            (lane = (pos, 8-dim slice)), B = the group's query heads (padded to 16) preloaded in registers;
//   softmax  online, base 2, one running maximum per head; the result lane (head, 4 positions) is already the A
//            operand layout of the second contraction;
//   output   O[head, dim] += P[head, pos] V_tile[pos, dim]: the V tile goes through LDS (rows padded to 272 bytes, so
//            the 2-byte transposed reads are conflict-free) to become the B operand; P is fed as bf16 high + low parts
//            (two MFMAs), which keeps the result within ~1e-5 of fp64.
// Waves are merged through LDS; with more than one split a second small kernel merges the splits.
#include <math.h>

#include "smc_internal.hpp"

namespace psmc {

namespace {
typedef short bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int vec16 __attribute__((ext_vector_type(4)));

constexpr int kAttnWaves = 2;             // waves per workgroup: small workgroups overlap each other's start-up and merge
constexpr int kTile = 16;                 // positions per MFMA tile
constexpr int kHeadsPad = 16;             // query heads of a group, padded to the MFMA width
constexpr float kLog2e = 1.4426950408889634f;

struct AttnSrc {
    const char* kA; const char* vA;   // dense: the K and the V tensor in buffer A; paged: their pools
    const char* kB; const char* vB;   // dense: the same tensors in buffer B
    const int32_t* parity;      // dense: which buffer holds row r
    const int32_t* table;       // paged: [R, M] page numbers
    const int32_t* done;        // termination flags (nullptr: no absorbing state): a terminated row is not read
    int P, M;                   // positions per page, pages per row
    int H, S;                   // KV heads, positions per row (dense)
};

__device__ __forceinline__ bf16x4 lo4(const vec16 v) { bf16x4 r; __builtin_memcpy(&r, &v, 8); return r; }
__device__ __forceinline__ bf16x4 hi4(const vec16 v) { bf16x4 r; __builtin_memcpy(&r, (const char*)&v + 8, 8); return r; }

// p = hi + lo with hi, lo representable in bf16 (hi by truncation, lo rounded to nearest even); returns the bit patterns
__device__ __forceinline__ void split_bf16(float p, unsigned& hi, unsigned& lo)
{
    const unsigned b = __float_as_uint(p);
    hi = b >> 16;
    const unsigned r = __float_as_uint(p - __uint_as_float(b & 0xFFFF0000u));
    lo = (r + 0x7FFFu + ((r >> 16) & 1u)) >> 16;
}
}  // namespace

// How positions are addressed: kDense = one contiguous run per (row, KV head) in the row's live buffer;
// kPagedAligned = paged with a page length that is a multiple of the tile (a tile lies in one page: one page number
// per tile, no per-lane division); kPagedAny = paged, any page length (page number and offset per lane).
enum { kDense = 0, kPagedAligned = 1, kPagedAny = 2 };

typedef const vec16 __attribute__((address_space(1)))* global_vec16_ptr;     // so that loads are global, not flat
__device__ __forceinline__ vec16 stream_load(const char* p) { return __builtin_nontemporal_load((global_vec16_ptr)p); }

// Partial result of one split for one query head: reference exponent, sum of weights, unnormalised output.
// Layout of the workspace: [row, query head, split, 2 + D] floats.
template <int D, int MODE>
__global__ __launch_bounds__(kAttnWaves* kWave) void attn_decode_kernel(
    AttnSrc src, const uint16_t* __restrict__ q, int Hq, int G, int len, float scale_log2, int n_splits, int tiles_per_split,
    float* __restrict__ partial, float* __restrict__ out)
{
    constexpr int NKL = D / 32;                 // 16-byte K loads per lane and tile
    constexpr int NDB = D / 16;                 // 16-dim blocks of the output
    constexpr int NVL = D / 32;                 // 16-byte V loads per lane and tile (16 positions x D x 2 bytes / 64 lanes / 16)
    constexpr int kRowBytes = D * 2 + 16;       // padded LDS row of a V tile
    constexpr int kPiecesPerRow = D / 8;        // 16-byte pieces per position
    constexpr int kPosBytes = D * 2;
    __shared__ __attribute__((aligned(16))) char sh_v[kAttnWaves][kTile * kRowBytes];
    __shared__ __attribute__((aligned(16))) float sh_alpha[kAttnWaves][kHeadsPad];
    __shared__ float sh_m[kAttnWaves][kHeadsPad], sh_l[kAttnWaves][kHeadsPad];
    __shared__ float sh_o[kAttnWaves][kHeadsPad][D];           // each wave's scaled output, summed when written out

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, j = lane >> 4;
    const int split = blockIdx.x % n_splits;
    const int head = (blockIdx.x / n_splits) % src.H;
    const int row = blockIdx.x / (n_splits * src.H);

    if (src.done && src.done[row]) {            // absorbing state (App. D): the particle's cache is not read, its output is 0
        for (int e = tid; e < G * D; e += kAttnWaves * kWave) {
            const int64_t hq = (int64_t)row * Hq + (int64_t)head * G + e / D;
            if (n_splits == 1) out[hq * D + e % D] = 0.f;
            else {
                float* rec = partial + (hq * n_splits + split) * (D + 2);
                if (e % D == 0) { rec[0] = 0.f; rec[1] = 1.f; }      // weight 1 on a zero vector: the merge gives 0
                rec[2 + e % D] = 0.f;
            }
        }
        return;
    }

    // the group's query heads as B operands: lane (head c, j) holds dims 32u + 8j .. + 7 of head c
    bf16x4 qb[2 * NKL];
    {
        const bool have = c < G;
        const uint16_t* qp = q + ((int64_t)row * Hq + (int64_t)head * G + (have ? c : 0)) * D;
#pragma unroll
        for (int u = 0; u < NKL; ++u) {
            vec16 v = *(const vec16*)(qp + 32 * u + 8 * j);
            if (!have) v = vec16{0u, 0u, 0u, 0u};
            qb[2 * u] = lo4(v);
            qb[2 * u + 1] = hi4(v);
        }
    }

    const int n_tiles = (len + kTile - 1) / kTile;
    const int tile_begin = split * tiles_per_split;
    const int tile_end = min(n_tiles, tile_begin + tiles_per_split);

    float m_run = -INFINITY;                    // running maximum (base-2 scores) of head c, equal in the 4 lanes of a head
    float l_run = 0.f;                          // sum of weights over this lane's own positions
    f32x4 acc[NDB];
#pragma unroll
    for (int t = 0; t < NDB; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Where the positions of this (row, KV head) live (see the MODE enumeration).  Page numbers are read one tile
    // ahead of the loads that need them, so the dependent load does not stall the stream.
    const int P = src.P;
    const int32_t* table_row = MODE == kDense ? nullptr : src.table + (int64_t)row * src.M;
    const int64_t page_stride = (int64_t)src.H * P * kPosBytes;
    const char* kbase; const char* vbase;
    if (MODE == kDense) {
        const bool in_b = src.parity[row] != 0;
        const int64_t off = ((int64_t)row * src.H + head) * src.S * kPosBytes;
        kbase = (in_b ? src.kB : src.kA) + off;
        vbase = (in_b ? src.vB : src.vA) + off;
    } else {
        kbase = src.kA + (int64_t)head * P * kPosBytes;
        vbase = src.vA + (int64_t)head * P * kPosBytes;
    }
    // lane-constant parts of the addresses inside a tile
    const int k_lane_off = c * kPosBytes + 16 * j;                              // position c of the tile, 16-byte piece j of a 64-byte run
    int v_lane_pos[NVL], v_lane_off[NVL];
#pragma unroll
    for (int u = 0; u < NVL; ++u) {
        const int piece = u * kWave + lane;
        v_lane_pos[u] = piece / kPiecesPerRow;
        v_lane_off[u] = (piece % kPiecesPerRow) * 16;
    }
    struct TilePages { int k; int v[NVL]; };
    auto lookup = [&](int tile, TilePages& tp) {
        const int p0 = tile * kTile;
        if (MODE == kPagedAligned) {
            tp.k = table_row[p0 / P];                                           // one page for the whole tile
        } else if (MODE == kPagedAny) {
            tp.k = table_row[min(p0 + c, len - 1) / P];
#pragma unroll
            for (int u = 0; u < NVL; ++u) tp.v[u] = table_row[min(p0 + v_lane_pos[u], len - 1) / P];
        }
    };
    // Positions past the end repeat the last valid one (their weights are masked to zero).
    auto load_tile = [&](int tile, const TilePages& tp, vec16 (&kd)[NKL], vec16 (&vd)[NVL]) {
        const int p0 = tile * kTile;
        const bool whole = p0 + kTile <= len;                                   // uniform: no clamping needed
        const char* kp; const char* vp[NVL];
        if (MODE == kDense) {
            const char* kt = kbase + (int64_t)p0 * kPosBytes;
            const char* vt = vbase + (int64_t)p0 * kPosBytes;
            kp = kt + (whole ? k_lane_off : min(c, len - 1 - p0) * kPosBytes + 16 * j);
#pragma unroll
            for (int u = 0; u < NVL; ++u)
                vp[u] = vt + (whole ? v_lane_pos[u] : min(v_lane_pos[u], len - 1 - p0)) * kPosBytes + v_lane_off[u];
        } else if (MODE == kPagedAligned) {
            const int64_t in_page = (int64_t)(p0 % P) * kPosBytes;
            const char* kt = kbase + tp.k * page_stride + in_page;
            const char* vt = vbase + tp.k * page_stride + in_page;
            kp = kt + (whole ? k_lane_off : min(c, len - 1 - p0) * kPosBytes + 16 * j);
#pragma unroll
            for (int u = 0; u < NVL; ++u)
                vp[u] = vt + (whole ? v_lane_pos[u] : min(v_lane_pos[u], len - 1 - p0)) * kPosBytes + v_lane_off[u];
        } else {
            const int kpos = min(p0 + c, len - 1);
            kp = kbase + tp.k * page_stride + (int64_t)(kpos % P) * kPosBytes + 16 * j;
#pragma unroll
            for (int u = 0; u < NVL; ++u) {
                const int vpos = min(p0 + v_lane_pos[u], len - 1);
                vp[u] = vbase + tp.v[u] * page_stride + (int64_t)(vpos % P) * kPosBytes + v_lane_off[u];
            }
        }
#pragma unroll
        for (int u = 0; u < NKL; ++u) kd[u] = stream_load(kp + 64 * u);        // dims 32u + 8j .. + 7 of the lane's position
#pragma unroll
        for (int u = 0; u < NVL; ++u) vd[u] = stream_load(vp[u]);
    };

    // One tile: scores, online softmax, output.  kc / vc hold the tile's K and V as loaded.
    auto process = [&](int tile, const vec16 (&kc)[NKL], const vec16 (&vc)[NVL]) {
        // scores of the tile: lane (head c, j) gets positions 4j .. 4j+3
        f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < NKL; ++u) {
            s = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(lo4(kc[u]), qb[2 * u], s, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(hi4(kc[u]), qb[2 * u + 1], s, 0, 0, 0);
        }
        float sv[4];
        float tmax = -INFINITY;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            sv[i] = (tile * kTile + 4 * j + i < len) ? s[i] * scale_log2 : -INFINITY;
            tmax = fmaxf(tmax, sv[i]);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float m_new = fmaxf(m_run, tmax);                 // finite: the tile has at least one valid position
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);   // 0 on the first tile (m_run = -inf)
        float p[4], psum = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) { p[i] = __builtin_amdgcn_exp2f(sv[i] - m_new); psum += p[i]; }
        l_run = l_run * alpha + psum;
        m_run = m_new;

        // rescale the output rows whose maximum moved; the factors travel through LDS (row = head 4j+i of this lane)
        if (__ballot(alpha != 1.f)) {
            if (j == 0) sh_alpha[wave][c] = alpha;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            const f32x4 a4 = *(const f32x4*)&sh_alpha[wave][4 * j];
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int t = 0; t < NDB; ++t) acc[t] *= a4;
        }

        // weights as A operands (head c, positions 4j..4j+3), bf16 high and low parts
        bf16x4 p_hi, p_lo;
        {
            unsigned h[4], l[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) split_bf16(p[i], h[i], l[i]);
            const unsigned ph[2] = {h[0] | (h[1] << 16), h[2] | (h[3] << 16)};
            const unsigned pl[2] = {l[0] | (l[1] << 16), l[2] | (l[3] << 16)};
            __builtin_memcpy(&p_hi, ph, 8);
            __builtin_memcpy(&p_lo, pl, 8);
        }

        // the V tile through LDS: written as rows, read as (4 consecutive positions of one dim)
        char* vt = sh_v[wave];
#pragma unroll
        for (int u = 0; u < NVL; ++u) *(vec16*)(vt + v_lane_pos[u] * kRowBytes + v_lane_off[u]) = vc[u];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int t = 0; t < NDB; ++t) {
            const char* col = vt + (4 * j) * kRowBytes + (16 * t + c) * 2;
            const unsigned v0 = *(const uint16_t*)(col), v1 = *(const uint16_t*)(col + kRowBytes);
            const unsigned v2 = *(const uint16_t*)(col + 2 * kRowBytes), v3 = *(const uint16_t*)(col + 3 * kRowBytes);
            const unsigned w[2] = {v0 | (v1 << 16), v2 | (v3 << 16)};
            bf16x4 vb;
            __builtin_memcpy(&vb, w, 8);
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(p_hi, vb, acc[t], 0, 0, 0);
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(p_lo, vb, acc[t], 0, 0, 0);
        }
        __builtin_amdgcn_wave_barrier();        // all lanes have read the tile before the next one overwrites it
    };

    // Software pipeline over this wave's tiles (tile, tile + 4, ...): while one tile is processed the next one's
    // loads are in flight and the page numbers of the one after are being read.  Unrolled by two so that the two
    // register buffers swap roles without copies.
    vec16 ka[NKL], va[NVL], kb[NKL], vb2[NVL];
    TilePages pg{};
    int tile = tile_begin + wave;
    if (tile < tile_end) {
        lookup(tile, pg);
        load_tile(tile, pg, ka, va);
        if (tile + kAttnWaves < tile_end) lookup(tile + kAttnWaves, pg);
    }
    while (tile < tile_end) {
        int next = tile + kAttnWaves;
        if (next < tile_end) {
            load_tile(next, pg, kb, vb2);
            if (next + kAttnWaves < tile_end) lookup(next + kAttnWaves, pg);
        }
        process(tile, ka, va);
        tile = next;
        if (tile >= tile_end) break;
        next = tile + kAttnWaves;
        if (next < tile_end) {
            load_tile(next, pg, ka, va);
            if (next + kAttnWaves < tile_end) lookup(next + kAttnWaves, pg);
        }
        process(tile, kb, vb2);
        tile = next;
    }

    // merge the waves: common reference per head, then sums and outputs
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    if (j == 0) { sh_m[wave][c] = m_run; sh_l[wave][c] = l_run; }
    __syncthreads();
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < kAttnWaves; ++w) M = fmaxf(M, sh_m[w][c]);
    if (j == 0) sh_alpha[wave][c] = m_run == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_run - M);   // a wave without tiles adds nothing
    __syncthreads();
    {
        const f32x4 f4 = *(const f32x4*)&sh_alpha[wave][4 * j];
#pragma unroll
        for (int t = 0; t < NDB; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) sh_o[wave][4 * j + i][16 * t + c] = acc[t][i] * f4[i];
    }
    __syncthreads();
    // head g < G: total weight L, then either the normalised output or this split's partial record
    for (int e = tid; e < G * D; e += kAttnWaves * kWave) {
        const int g = e / D, d = e % D;
        float Mg = -INFINITY;
#pragma unroll
        for (int w = 0; w < kAttnWaves; ++w) Mg = fmaxf(Mg, sh_m[w][g]);
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < kAttnWaves; ++w) L += sh_l[w][g] * sh_alpha[w][g];
        float o = 0.f;
#pragma unroll
        for (int w = 0; w < kAttnWaves; ++w) o += sh_o[w][g][d];
        const int64_t hq = (int64_t)row * Hq + (int64_t)head * G + g;
        if (n_splits == 1) {
            out[hq * D + d] = o / L;
        } else {
            float* rec = partial + (hq * n_splits + split) * (D + 2);
            if (d == 0) { rec[0] = Mg; rec[1] = L; }
            rec[2 + d] = o;
        }
    }
}

// Merges the splits of one (row, query head): out = sum_s o_s 2^(M_s - M) / sum_s L_s 2^(M_s - M).
template <int D>
__global__ __launch_bounds__(D) void attn_combine_kernel(const float* __restrict__ partial, int n_splits, float* __restrict__ out)
{
    const int64_t hq = blockIdx.x;
    const int d = threadIdx.x;
    const float* rec = partial + hq * n_splits * (D + 2);
    float M = -INFINITY;
    for (int s = 0; s < n_splits; ++s) M = fmaxf(M, rec[s * (D + 2)]);
    float L = 0.f, o = 0.f;
    for (int s = 0; s < n_splits; ++s) {
        const float f = __builtin_amdgcn_exp2f(rec[s * (D + 2)] - M);
        L += rec[s * (D + 2) + 1] * f;
        o += rec[s * (D + 2) + 2 + d] * f;
    }
    out[hq * D + d] = o / L;
}

}  // namespace psmc

using namespace psmc;

namespace {
constexpr int kMaxAttnSplits = 16;
}

extern "C" {

size_t smc_attn_workspace_bytes(const smc_config* cfg, int32_t n_q_heads)
{
    if (!cfg || cfg->kv_tensors < 2 || n_q_heads < 1 || cfg->kv_H < 1 || n_q_heads % cfg->kv_H != 0) return 0;
    if (cfg->kv_D != 64 && cfg->kv_D != 128) return 0;
    return (size_t)cfg->B * cfg->N * n_q_heads * kMaxAttnSplits * (cfg->kv_D + 2) * sizeof(float);
}

smc_status smc_attn_decode(smc_ctx* ctx, int32_t k_tensor, int32_t v_tensor, const void* d_q, int32_t n_q_heads, int32_t len,
                           float scale, void* d_workspace, size_t workspace_bytes, float* d_out)
{
    if (!ctx || !d_q || !d_out || !d_workspace) return SMC_E_NULL;
    const auto& cfg = ctx->cfg;
    if (cfg.kv_tensors < 1 || k_tensor < 0 || v_tensor < 0 || k_tensor >= cfg.kv_tensors || v_tensor >= cfg.kv_tensors)
        return SMC_E_RANGE;
    if (cfg.kv_elem_bytes != 2) return SMC_E_DTYPE;
    if (cfg.kv_D != 64 && cfg.kv_D != 128) return SMC_E_SHAPE;
    if (n_q_heads < 1 || n_q_heads % cfg.kv_H != 0 || n_q_heads / cfg.kv_H > kHeadsPad) return SMC_E_SHAPE;
    if (len < 1 || len > cfg.kv_S) return SMC_E_RANGE;
    if (!(scale > 0.f) || !(scale < 3.0e38f)) return SMC_E_RANGE;
    if (((uintptr_t)d_q & 15u) != 0 || ((uintptr_t)d_out & 15u) != 0 || ((uintptr_t)d_workspace & 15u) != 0) return SMC_E_ALIGN;
    if (workspace_bytes < smc_attn_workspace_bytes(&cfg, n_q_heads)) return SMC_E_SHAPE;
    const bool paged = ctx->paged.bound != 0;
    if (!paged && !ctx->kv_bound) return SMC_E_STATE;
    if (paged && len > ctx->paged.len) return SMC_E_RANGE;       // positions that were never appended have no page

    AttnSrc src{};
    if (paged) {
        src.kA = (const char*)ctx->h_pools[k_tensor]; src.vA = (const char*)ctx->h_pools[v_tensor];
    } else {
        src.kA = (const char*)ctx->h_kvA[k_tensor]; src.vA = (const char*)ctx->h_kvA[v_tensor];
        src.kB = (const char*)ctx->h_kvB[k_tensor]; src.vB = (const char*)ctx->h_kvB[v_tensor];
    }
    src.parity = ctx->ws.parity;
    src.done = cfg.eos_id >= 0 ? ctx->ws.done : nullptr;
    src.table = paged ? ctx->paged.table : nullptr;
    src.P = paged ? ctx->paged.P : 1;
    src.M = paged ? ctx->paged.M : 0;
    src.H = cfg.kv_H; src.S = cfg.kv_S;

    const int G = n_q_heads / cfg.kv_H;
    const int n_tiles = (len + kTile - 1) / kTile;
    const int64_t units = (int64_t)ctx->R * cfg.kv_H;
    // Every split pays a fixed start-up and merge cost and more than one needs the merge launch, so a row's positions
    // are split only when there are fewer than two workgroups per compute unit (measured: 512 workgroups of cfg2's
    // shape run as fast unsplit as split in two), and never below four tiles per wave.
    const int64_t slots = 2 * (int64_t)ctx->n_cus;
    int n_splits = (int)((slots + units - 1) / units);
    n_splits = n_splits < 1 ? 1 : n_splits;
    if (n_splits > kMaxAttnSplits) n_splits = kMaxAttnSplits;
    const int max_by_work = n_tiles / (4 * kAttnWaves);
    if (n_splits > max_by_work) n_splits = max_by_work < 1 ? 1 : max_by_work;
    const int tiles_per_split = (n_tiles + n_splits - 1) / n_splits;
    n_splits = (n_tiles + tiles_per_split - 1) / tiles_per_split;            // no empty split

    const dim3 grid((unsigned)(units * n_splits)), block(kAttnWaves * kWave);
    const float scale_log2 = scale * kLog2e;
    const int mode = !paged ? kDense : (ctx->paged.P % kTile == 0 ? kPagedAligned : kPagedAny);
    {
        ScopedKernelTimer timer(ctx, 3);
#define PSMC_ATTN(DD, MM) hipLaunchKernelGGL((attn_decode_kernel<DD, MM>), grid, block, 0, ctx->stream, src, (const uint16_t*)d_q, \
                                             n_q_heads, G, len, scale_log2, n_splits, tiles_per_split, (float*)d_workspace, d_out)
        if (cfg.kv_D == 128) {
            if (mode == kDense) PSMC_ATTN(128, kDense); else if (mode == kPagedAligned) PSMC_ATTN(128, kPagedAligned); else PSMC_ATTN(128, kPagedAny);
        } else {
            if (mode == kDense) PSMC_ATTN(64, kDense); else if (mode == kPagedAligned) PSMC_ATTN(64, kPagedAligned); else PSMC_ATTN(64, kPagedAny);
        }
#undef PSMC_ATTN
    }
    if (n_splits > 1) {
        const dim3 cgrid((unsigned)((int64_t)ctx->R * n_q_heads));
        if (cfg.kv_D == 128)
            hipLaunchKernelGGL((attn_combine_kernel<128>), cgrid, dim3(128), 0, ctx->stream, (const float*)d_workspace, n_splits, d_out);
        else
            hipLaunchKernelGGL((attn_combine_kernel<64>), cgrid, dim3(64), 0, ctx->stream, (const float*)d_workspace, n_splits, d_out);
    }
    return hipGetLastError() == hipSuccess ? SMC_OK : SMC_E_HIP;
}

}  // extern "C"
