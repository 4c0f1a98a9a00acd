// Winograd F(4x4, 3x3) in one kernel: input transform, the 36 products on the matrix cores and the output transform
// without the transformed input and the products ever reaching memory (Section 4 lists Winograd among the implementations
// an operator chooses from; Appendix D: workspace against time -- this is the small-workspace end: the workspace holds the
// transformed filters only).
//
//   Y = A^T [ (G g G^T) .* (B^T d B) ] A     per 6x6 input tile d, 3x3 filter g, 4x4 output tile Y (matrices: winograd.hip)
//
// A workgroup (four waves, one per SIMD) owns 32 tiles x 64 output channels for all 36 positions z of the transformed
// tile: wave w keeps the nine products z = 9w .. 9w+8 as 9 x 2 accumulator blocks of 32x32 (288 registers per lane).  The
// reduction runs over the input channels in chunks of 8:
//   * every thread loads the 6x6 patch of one (tile, channel) of the next chunk straight from the activation tensor
//     (neighbouring tiles overlap by two rows / columns; the overlap is served by the caches), transforms it in registers
//     and leaves V[z][tile][c] in one of two LDS buffers;
//   * the A operand of v_mfma_f32_32x32x2_f32 (lane -> tile l % 32, channel l / 32) is one LDS word per lane; the B
//     operand comes from the transformed filters, which the filter kernel below stores in exactly the order the lanes
//     read them (one 16-byte load per lane covers the four steps of a chunk), three positions ahead of their use.
// After the last chunk the accumulators go through LDS in two halves of 32 channels (36 x 32 x 32 floats each), and one
// thread per (tile, channel) applies A^T . A and writes the 4x4 outputs, optionally added to what is there (a second
// consumer's gradient) or followed by a BatchNorm apply step (recomputation).
//
// Traffic: the input once per block of 64 output channels (plus the tile overlap where the caches miss), the output once,
// the transformed filters from L2.  With many channels the input passes and the filter stream (36 x 64 floats per input
// channel and workgroup) cost more than the workspace form's large GEMM tiles save; the graph offers this form where it
// was measured to be faster.
#include "bn_affine.hpp"
#include "buffer_addr.hpp"
#include "kernels.hpp"

namespace monet {

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int FT = 32;            // tiles per workgroup
constexpr int FK = 64;            // output channels per workgroup
constexpr int FC = 8;             // reduction channels per chunk
constexpr int FUSED_CUS = 256;    // one workgroup per CU (LDS)
constexpr int VROW = FC + 1;      // row of V[z][tile][.] in LDS, padded: 32 tiles x 9 words hit 32 different banks
constexpr int MROW = 33;          // row of M[z][tile][.] in LDS
constexpr int LDS_FLOATS = 36 * FT * MROW;               // 152 064 bytes; the two V buffers take the first 82 944
static_assert(2 * 36 * FT * VROW <= LDS_FLOATS, "V buffers must fit");

// The one-dimensional maps of F(4, 3).  On this chip fp32 matrix instructions and ordinary vector arithmetic exclude each
// other on a SIMD (measured: every vector instruction costs the matrix pipe about 4.7 cycles, whichever wave issues it),
// so the transforms are written for the fewest instructions: B^T in twelve multiply-adds
//   B^T = [4 0 -5 0 1 0; 0 -4 -4 1 1 0; 0 4 -4 -1 1 0; 0 -2 -1 2 1 0; 0 2 -1 -2 1 0; 0 4 0 -5 0 1]
__device__ inline void f4_bt(float v0, float v1, float v2, float v3, float v4, float v5, float (&o)[6]) {
    const float p = __builtin_fmaf(-4.0f, v2, v4), q = __builtin_fmaf(-4.0f, v1, v3);
    const float r = v4 - v2, t = v3 - v1;
    o[0] = __builtin_fmaf(4.0f, v0, __builtin_fmaf(-5.0f, v2, v4));
    o[1] = p + q;
    o[2] = p - q;
    o[3] = __builtin_fmaf(2.0f, t, r);
    o[4] = __builtin_fmaf(-2.0f, t, r);
    o[5] = __builtin_fmaf(4.0f, v1, __builtin_fmaf(-5.0f, v3, v5));
}
__device__ inline void f4_g(float g0, float g1, float g2, float (&o)[6]) {
    o[0] = 0.25f * g0;
    o[1] = (-1.0f / 6.0f) * (g0 + g1 + g2);
    o[2] = (-1.0f / 6.0f) * (g0 - g1 + g2);
    o[3] = (1.0f / 24.0f) * g0 + (1.0f / 12.0f) * g1 + (1.0f / 6.0f) * g2;
    o[4] = (1.0f / 24.0f) * g0 - (1.0f / 12.0f) * g1 + (1.0f / 6.0f) * g2;
    o[5] = g2;
}
//   A^T = [1 1 1 1 1 0; 0 1 -1 2 -2 0; 0 1 1 4 4 0; 0 1 -1 8 -8 1]
__device__ inline void f4_at(float m0, float m1, float m2, float m3, float m4, float m5, float (&o)[4]) {
    const float p = m1 + m2, q = m1 - m2, r = m3 + m4, t = m3 - m4;
    o[0] = m0 + p + r;
    o[1] = __builtin_fmaf(2.0f, t, q);
    o[2] = __builtin_fmaf(4.0f, r, p);
    o[3] = __builtin_fmaf(8.0f, t, q) + m5;
}

// Transformed filters in the order the matrix-core lanes read them:
//   Up[z][out / 32][red / 8][lane][j],  lane = 32 * (red % 2) + out % 32,  j = (red % 8) / 2
// `out` runs over the output channels padded to a multiple of 64 (zeros), `red` over the reduction channels.
// ADJ: forward pass (out = K, red = C) or input gradient (out = C, red = K, filter turned by 180 degrees).
template <bool ADJ>
__global__ __launch_bounds__(256) void wino4_filter_fused_kernel(const float *__restrict__ w, float *__restrict__ Up, int K, int C, int out_pad) {
    const int outc = ADJ ? C : K, red = ADJ ? K : C;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)out_pad * red) return;
    const int o = (int)(idx / red), c = (int)(idx % red);
    float g[3][3];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s)
            g[r][s] = o >= outc ? 0.0f : (ADJ ? w[((int64_t)c * 9 + (2 - r) * 3 + (2 - s)) * C + o] : w[((int64_t)o * 9 + r * 3 + s) * C + c]);
    float t[3][6];      // t[s][a] = (G g)[a][s]
#pragma unroll
    for (int s = 0; s < 3; ++s) f4_g(g[0][s], g[1][s], g[2][s], t[s]);
    const int nch = red / FC, o32 = out_pad / 32;
    const int lane = 32 * (c & 1) + (o & 31), j = (c & 7) >> 1;
#pragma unroll
    for (int a = 0; a < 6; ++a) {
        float u[6];
        f4_g(t[0][a], t[1][a], t[2][a], u);
#pragma unroll
        for (int b = 0; b < 6; ++b) {
            const int z = 6 * a + b;
            Up[((((int64_t)z * o32 + (o >> 5)) * nch + (c >> 3)) * 64 + lane) * 4 + j] = u[b];
        }
    }
}


struct FusedGeom {
    int N, H, W, th, tw;
    int64_t T;          // tiles
    int red, outc;      // reduction / output channels
    int nch;            // red / 8
    int kblocks;        // ceil(outc / 64)
    int64_t items;      // ceil(T / 32) * kblocks
    // Items [main_items, items) are worked as two half items of 32 output channels each (the ragged last round of a launch
    // with few items: a half item takes about 0.6 of a whole one, and twice as many CUs take part).  main_items is a
    // multiple of 8; main_items == items: no item is halved.
    int64_t main_items;
};

// What a patch lane knows about its (tile, channel): byte offsets of the six patch columns / rows (clamped into the map) and
// which of them exist.  Patch element (a, b) of chunk ch sits at byte x + coff[b] + roff[a] + 32 * ch; the host checks that
// the tensor has fewer than 2^32 bytes.
struct PatchLane {
    unsigned coff[6], roff[6];      // column b: (image, row 0, column 4 * tj + b - 1, channel pc); row a: row 4 * ti + a - 1
    unsigned rowok, colok;
};

// tinfo[tile] = {byte offset of output element (image, 4 * ti, 4 * tj, channel 0), rows | columns << 8 of the 4x4 output tile
// that lie inside the map (0 for a tile beyond the last one)}: written once per tile by the patch lane of channel 0, read by
// the output transform, which so needs no division.
__device__ __forceinline__ PatchLane patch_lane(const FusedGeom &gm, int64_t tb, int ptid, unsigned (*tinfo)[2]) {
    PatchLane pl;
#pragma unroll
    for (int a = 0; a < 6; ++a) pl.coff[a] = pl.roff[a] = 0;
    pl.rowok = pl.colok = 0;
    const int pc = ptid & 7, pt = ptid >> 3;
    const unsigned t = (unsigned)(tb * FT) + pt;      // the host checks that there are fewer than 2^31 tiles
    unsigned out_off = 0, extent = 0;
    if (t < (unsigned)gm.T) {
        const unsigned tj = t % (unsigned)gm.tw, r = t / (unsigned)gm.tw;
        const unsigned ti = r % (unsigned)gm.th, n = r / (unsigned)gm.th;
        const int h0 = 4 * (int)ti - 1, w0 = 4 * (int)tj - 1;
        const int64_t e = ((int64_t)n * gm.H * gm.W) * gm.red + pc;
#pragma unroll
        for (int a = 0; a < 6; ++a) {
            if ((unsigned)(h0 + a) < (unsigned)gm.H) pl.rowok |= 1u << a;
            if ((unsigned)(w0 + a) < (unsigned)gm.W) pl.colok |= 1u << a;
            const int hc = min(max(h0 + a, 0), gm.H - 1), wc = min(max(w0 + a, 0), gm.W - 1);
            pl.roff[a] = (unsigned)((int64_t)hc * gm.W * gm.red * 4);
            pl.coff[a] = (unsigned)((e + (int64_t)wc * gm.red) * 4);
        }
        out_off = (unsigned)((((int64_t)n * gm.H + 4 * ti) * gm.W + 4 * tj) * gm.outc * 4);
        extent = (unsigned)min(4, gm.H - 4 * (int)ti) | ((unsigned)min(4, gm.W - 4 * (int)tj) << 8);
    }
    if (pc == 0) {
        tinfo[pt][0] = out_off;
        tinfo[pt][1] = extent;
    }
    return pl;
}

// The reduction loop of one wave: NZ positions z0 .. z0 + NZ - 1 of the 32 x 64 tile; PATCH: this wave also loads and
// transforms the input patches (one (tile, channel) per lane and chunk); INTERIOR: all of the wave's patches lie inside
// the map (nothing to clamp, nothing to zero); HALF: a half item, only the block of 32 output channels ob (acc[.][0]); else
// the blocks ob and ob + 1.
template <int NZ, bool PATCH, bool INTERIOR, bool HALF>
__device__ __forceinline__ void fused_reduce(const float *__restrict__ x, const float *__restrict__ Up, float *lds, const FusedGeom &gm, int ob,
                                             int z0, int ptid, int lane, const PatchLane &pl, floatx16 (&acc)[5][2]) {
    const int l32 = lane & 31, g = lane >> 5;
    const int nch = gm.nch;
    const int pc = ptid & 7, pt = ptid >> 3;
    float d[36];
    // interior patches: row a - 1 relative to the tile's first output row goes into the scalar offset (the descriptor starts
    // one image row before the tensor; only offsets that lead back into it are used)
    const unsigned rowbytes = (unsigned)gm.W * gm.red * 4;
    const __amdgpu_buffer_rsrc_t rx = buffer_of(INTERIOR ? (const char *)x - rowbytes : (const char *)x);
    auto load_patch = [&](int ch) {
        const unsigned cbytes = (unsigned)ch * (FC * 4);
        if (INTERIOR) {
            unsigned vb[6];
#pragma unroll
            for (int b = 0; b < 6; ++b) vb[b] = pl.coff[b] + pl.roff[1] + cbytes;
#pragma unroll
            for (int a = 0; a < 6; ++a)
#pragma unroll
                for (int b = 0; b < 6; ++b) d[a * 6 + b] = buffer_load(rx, vb[b], a * rowbytes);
        } else {
#pragma unroll
            for (int a = 0; a < 6; ++a)
#pragma unroll
                for (int b = 0; b < 6; ++b) d[a * 6 + b] = buffer_load(rx, pl.coff[b] + pl.roff[a], cbytes);
        }
    };
    auto transform_store = [&](float *V) {
        if (!INTERIOR) {
#pragma unroll
            for (int a = 0; a < 6; ++a)
#pragma unroll
                for (int b = 0; b < 6; ++b)
                    if (!((pl.rowok >> a) & (pl.colok >> b) & 1u)) d[a * 6 + b] = 0.0f;
        }
        float m[6][6];      // m[b][a] = (B^T d)[a][b]
#pragma unroll
        for (int b = 0; b < 6; ++b) f4_bt(d[b], d[6 + b], d[12 + b], d[18 + b], d[24 + b], d[30 + b], m[b]);
#pragma unroll
        for (int a = 0; a < 6; ++a) {
            float o[6];
            f4_bt(m[0][a], m[1][a], m[2][a], m[3][a], m[4][a], m[5][a], o);
#pragma unroll
            for (int b = 0; b < 6; ++b) V[((6 * a + b) * FT + pt) * VROW + pc] = o[b];
        }
    };

    // ---- B operands: position z0 + zi, channel blocks ob and (a whole item) ob + 1, chunk ch.  Loads return in the order they
    // were issued, so they are issued in the order of their use: the positions of chunk ch + 1 are requested while chunk ch
    // is multiplied (each into the registers its predecessor just left), after the patch of chunk ch + 1, which is
    // requested first and used last.
    const int o32 = gm.kblocks * 2;
    const __amdgpu_buffer_rsrc_t ru = buffer_of(Up);
    const unsigned lane16 = (unsigned)lane * 16u;
    const unsigned zbytes = (unsigned)o32 * nch * 1024u, hbytes = (unsigned)nch * 1024u;      // the host checks the workspace size
    const unsigned b0bytes = ((unsigned)z0 * o32 + (unsigned)ob) * nch * 1024u;
    f4 bq[NZ][2];
    auto load_b = [&](int zi, int ch) {
        const unsigned so = b0bytes + zi * zbytes + (unsigned)ch * 1024u;
        bq[zi][0] = buffer_load4(ru, lane16, so);
        if (!HALF) bq[zi][1] = buffer_load4(ru, lane16, so + hbytes);
    };

    if (PATCH) load_patch(0);
#pragma unroll
    for (int zi = 0; zi < NZ; ++zi) load_b(zi, 0);
    if (PATCH) {
        transform_store(lds);
        load_patch(nch > 1 ? 1 : 0);
    }
    __syncthreads();

    for (int ch = 0; ch < nch; ++ch) {
        const float *Vcur = lds + (ch & 1) * (36 * FT * VROW);
        float *Vnext = lds + ((ch + 1) & 1) * (36 * FT * VROW);
        // the last chunks request operands that exist (their own) instead of branching around the requests; nothing reads them
        const int nx = ch + 1 < nch ? ch + 1 : ch, nx2 = ch + 2 < nch ? ch + 2 : nch - 1;
        // A patch wave transforms first (the patch of chunk ch + 1 was requested a whole chunk ago; V[next] was last read
        // before the barrier that ended chunk ch - 1), so that its arithmetic runs beside the other wave's matrix-core
        // work, then requests the patch of chunk ch + 2, then multiplies.  The scheduler must not move requests towards
        // their use (it would, to save registers): the order of the sections below is the order of issue.
        if (PATCH) {
            transform_store(Vnext);
            __builtin_amdgcn_sched_barrier(0);
            load_patch(nx2);
        }
        __builtin_amdgcn_sched_barrier(0);
        const float *vp = Vcur + (z0 * FT + l32) * VROW + g;
        float a0 = vp[0], a1 = vp[2], a2 = vp[4], a3 = vp[6];
#pragma unroll
        for (int zi = 0; zi < NZ; ++zi) {
            const float c0 = a0, c1 = a1, c2 = a2, c3 = a3;
            if (zi + 1 < NZ) {      // A operands of the next position, read while this one multiplies
                const float *vn = vp + (zi + 1) * (FT * VROW);
                a0 = vn[0]; a1 = vn[2]; a2 = vn[4]; a3 = vn[6];
            }
            __builtin_amdgcn_sched_barrier(0);
            acc[zi][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(c0, bq[zi][0].x, acc[zi][0], 0, 0, 0);
            if (!HALF) acc[zi][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(c0, bq[zi][1].x, acc[zi][1], 0, 0, 0);
            acc[zi][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(c1, bq[zi][0].y, acc[zi][0], 0, 0, 0);
            if (!HALF) acc[zi][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(c1, bq[zi][1].y, acc[zi][1], 0, 0, 0);
            acc[zi][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(c2, bq[zi][0].z, acc[zi][0], 0, 0, 0);
            if (!HALF) acc[zi][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(c2, bq[zi][1].z, acc[zi][1], 0, 0, 0);
            acc[zi][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(c3, bq[zi][0].w, acc[zi][0], 0, 0, 0);
            if (!HALF) acc[zi][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(c3, bq[zi][1].w, acc[zi][1], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            load_b(zi, nx);      // into the registers the products above have just read
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();      // V[next] complete; every wave is done reading V[cur]
    }
}

// Output transform of one (tile, channel): the 36 products from LDS, A^T . A, the 16 outputs to memory.
// EPI: 0 plain store, 1 added to what is there, 2 followed by the BatchNorm multiply-add.  WHOLE: every output of the tile
// lies inside the map and the channel exists (no store needs a test).
template <int EPI, bool WHOLE>
__device__ __forceinline__ void fused_output(const float *mp, __amdgpu_buffer_rsrc_t ry, unsigned voff, unsigned orow, unsigned obytes, int nr,
                                             int nc, float bn_a, float bn_b, int relu, __amdgpu_buffer_rsrc_t ry2, bool two,
                                             unsigned *mask32, int lane) {
    float s[6][4];      // s[b][a] = (A^T m)[a][b]
#pragma unroll
    for (int b = 0; b < 6; ++b) {
        float m[6];
#pragma unroll
        for (int a = 0; a < 6; ++a) m[a] = mp[(6 * a + b) * (FT * MROW)];
        f4_at(m[0], m[1], m[2], m[3], m[4], m[5], s[b]);
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        float o[4];
        f4_at(s[0][a], s[1][a], s[2][a], s[3][a], s[4][a], s[5][a], o);
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const unsigned so = a * orow + b * obytes;
            const bool here = WHOLE || (a < nr && b < nc);
            if (EPI == 2 && mask32) {      // uniform over the wave
                // the sign code of the ReLU: the 32 lanes of a half wave hold 32 consecutive channels of one position, half
                // a word of the code; its first lane writes it
                const float e = bn_affine(o[b], bn_a, bn_b);
                const bool pass = here && (relu == 2 ? (e > 0.0f && e < 6.0f) : e > 0.0f);
                const unsigned long long word = __ballot(pass);
                const unsigned half = lane < 32 ? (unsigned)word : (unsigned)(word >> 32);
                if ((lane & 31) == 0 && here) mask32[(voff + so) >> 7] = half;
            }
            if (here) {
                float v = o[b];
                if (EPI == 1) v += buffer_load(ry, voff, so);
                if (EPI == 2) v = bn_affine(v, bn_a, bn_b);
                if (EPI == 2 && relu) {
                    const float rv = relu_clamp(v, relu);
                    if (two) buffer_store(ry2, voff, so, rv);
                    else v = rv;
                }
                buffer_store(ry, voff, so, v);
            }
        }
    }
}

// Eight waves, two per SIMD: waves 0-3 multiply five positions each (z = 5w ..), waves 4-7 four positions each
// (z = 20 + 4(w - 4) ..) and transform the input patches, so that on every SIMD the transform arithmetic of one wave runs
// beside the matrix-core work of the other.  ADJ only names the use in profiles (forward pass / input gradient).
template <bool ADJ, int EPI>
__global__ __launch_bounds__(512) void wino4_fused_kernel(const float *__restrict__ x, const float *__restrict__ Up, float *y, FusedGeom gm,
                                                          BnAffine bn) {
    __shared__ float lds[LDS_FLOATS];
    __shared__ unsigned tinfo[FT][2];
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // the same for the whole wave: kept in a scalar register
    // Work item: hardware deals workgroups to the 8 XCDs in turn; item = (id mod 8) * (grid / 8) + id / 8 gives each XCD a
    // contiguous share, so that neighbouring tile rows (shared halo) and the channel blocks of one tile range (same input)
    // meet in one L2.  The grid is a multiple of 8; items beyond the last one do nothing.
    // Every XCD takes its share of the whole items first, then its share of the half items, so that the short ones come
    // last everywhere.
    const int64_t id = blockIdx.x, xcd = id & 7, idx = id >> 3;
    const int64_t pm = gm.main_items >> 3;
    int64_t item;
    int nh = 2, hsel = 0;          // blocks of 32 output channels this workgroup computes; the first of them within the item
    if (gm.main_items == gm.items) {      // no item is halved: a contiguous share of the items per XCD
        item = xcd * ((int64_t)gridDim.x >> 3) + idx;
        if (item >= gm.items) return;
    } else if (idx < pm) {
        item = xcd * pm + idx;
    } else {
        const int64_t nhalf = (gm.items - gm.main_items) * 2, pt = (nhalf + 7) >> 3;
        const int64_t j = xcd * pt + (idx - pm);
        if (idx - pm >= pt || j >= nhalf) return;
        item = gm.main_items + (j >> 1);
        nh = 1;
        hsel = (int)(j & 1);
    }
    const int kb = (int)(item % gm.kblocks);
    const int64_t tb = item / gm.kblocks;
    const int ob = 2 * kb + hsel;
    if (ob * 32 >= gm.outc) return;      // the second half of a last, half-empty channel block (uniform over the workgroup)

    floatx16 acc[5][2];
#pragma unroll
    for (int zi = 0; zi < 5; ++zi)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[zi][h][i] = 0.0f;
    const bool heavy = wave < 4;
    const int z0 = heavy ? 5 * wave : 20 + 4 * (wave - 4), nz = heavy ? 5 : 4;
    if (heavy) {
        if (nh == 2) fused_reduce<5, false, false, false>(x, Up, lds, gm, ob, z0, 0, lane, PatchLane{}, acc);
        else fused_reduce<5, false, false, true>(x, Up, lds, gm, ob, z0, 0, lane, PatchLane{}, acc);
    } else {
        const PatchLane pl = patch_lane(gm, tb, tid - 256, tinfo);      // tinfo is complete at the loop's first barrier
        // uniform over the wave; every version of the loop meets the workgroup's barriers the same number of times
        const bool interior = __all(pl.rowok == 0x3fu && pl.colok == 0x3fu);
        if (nh == 2) {
            if (interior) fused_reduce<4, true, true, false>(x, Up, lds, gm, ob, z0, tid - 256, lane, pl, acc);
            else fused_reduce<4, true, false, false>(x, Up, lds, gm, ob, z0, tid - 256, lane, pl, acc);
        } else {
            if (interior) fused_reduce<4, true, true, true>(x, Up, lds, gm, ob, z0, tid - 256, lane, pl, acc);
            else fused_reduce<4, true, false, true>(x, Up, lds, gm, ob, z0, tid - 256, lane, pl, acc);
        }
    }

    // ---- output transform, 32 channels at a time: thread = (channel ok_ of the half, tiles oq and oq + 16).  Output element
    // (a, b) of a tile sits at byte y + [(a * W + b) * outc * 4] + voff: the bracket is scalar, voff the thread's own 32-bit
    // offset (tile + channel); the host checks that the output has fewer than 2^32 bytes.
    const int ok_ = tid & 31, oq = tid >> 5;
    const unsigned obytes = (unsigned)gm.outc * 4, orow = (unsigned)gm.W * obytes;
    const __amdgpu_buffer_rsrc_t ry = buffer_of(y);
    const bool two = EPI == 2 && bn.relu && bn.relu_out != nullptr;           // ReLU output beside the BatchNorm's
    const __amdgpu_buffer_rsrc_t ry2 = buffer_of(two ? bn.relu_out : y);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int kout = (ob + h) * 32 + ok_;
        if (h >= nh || (ob + h) * 32 >= gm.outc) break;       // uniform over the workgroup
        if (h) __syncthreads();                        // the first half has been read
#pragma unroll
        for (int zi = 0; zi < 5; ++zi)
            if (zi < nz) {
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    lds[((z0 + zi) * FT + 8 * (i >> 2) + 4 * g + (i & 3)) * MROW + l32] = acc[zi][h][i];
            }
        __syncthreads();
        float bn_a = 1.0f, bn_b = 0.0f;
        if (EPI == 2 && kout < gm.outc) bn_affine_coeffs(bn.gamma, bn.beta, bn.stats, gm.outc, kout, bn_a, bn_b);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int tl = oq + 16 * q;
            const unsigned voff = tinfo[tl][0] + (unsigned)kout * 4u;
            unsigned ext = tinfo[tl][1];
            if (kout >= gm.outc) ext = 0;
            const float *mp = lds + tl * MROW + ok_;
            unsigned *mask32 = EPI == 2 && bn.relu ? (unsigned *)bn.mask : nullptr;
            if (__all(ext == (4u | (4u << 8)))) fused_output<EPI, true>(mp, ry, voff, orow, obytes, 4, 4, bn_a, bn_b, bn.relu, ry2, two, mask32, lane);      // uniform over the wave
            else fused_output<EPI, false>(mp, ry, voff, orow, obytes, (int)(ext & 0xff), (int)(ext >> 8), bn_a, bn_b, bn.relu, ry2, two, mask32, lane);
        }
    }
}

}  // namespace

bool winograd_fused_applies(const ConvShape &cs, bool adjoint) {
    if (cs.R != 3 || cs.S != 3 || cs.stride != 1 || cs.pad != 1) return false;
    const int red = adjoint ? cs.K : cs.C, out = adjoint ? cs.C : cs.K;
    return red % FC == 0 && out >= 1;
}

size_t winograd_fused_workspace_bytes(const ConvShape &cs, bool adjoint) {
    const int red = adjoint ? cs.K : cs.C, out = adjoint ? cs.C : cs.K;
    return (size_t)36 * ((out + FK - 1) / FK * FK) * red * sizeof(float);
}

void conv_winograd_fused(hipStream_t st, const float *in, const float *w, float *out, const ConvShape &cs, bool adjoint, bool accumulate,
                         float *ws, size_t ws_bytes, const BnAffine *affine) {
    if (affine && (adjoint || accumulate || !affine->gamma || !affine->beta || !affine->stats))
        throw KernelError("conv_winograd_fused: a BatchNorm apply step goes with the forward form, without accumulation, and needs all coefficients");
    if (affine && affine->mask && (!affine->relu || cs.K % 64))
        throw KernelError("conv_winograd_fused: a sign code in the epilogue needs the ReLU and K % 64 == 0");
    if (!winograd_fused_applies(cs, adjoint))
        throw KernelError("conv_winograd_fused: needs a 3x3 / stride 1 / pad 1 layer whose reduction channels are a multiple of 8");
    if (!ws || ws_bytes < winograd_fused_workspace_bytes(cs, adjoint))
        throw KernelError("conv_winograd_fused: workspace too small for the transformed filters");
    FusedGeom gm;
    gm.N = cs.N; gm.H = cs.H; gm.W = cs.W;
    gm.th = (cs.H + 3) / 4; gm.tw = (cs.W + 3) / 4;
    gm.T = (int64_t)cs.N * gm.th * gm.tw;
    gm.red = adjoint ? cs.K : cs.C;
    gm.outc = adjoint ? cs.C : cs.K;
    gm.nch = gm.red / FC;
    gm.kblocks = (gm.outc + FK - 1) / FK;
    gm.items = (gm.T + FT - 1) / FT * gm.kblocks;
    // the ragged last round: at most half a round of whole items beyond a multiple of the CU count becomes at most one
    // round of half items
    gm.main_items = gm.items;
    if (gm.items % FUSED_CUS && gm.items % FUSED_CUS <= FUSED_CUS / 2) gm.main_items = gm.items - gm.items % FUSED_CUS;      // also a launch of at most half a round
    const int64_t grid = gm.main_items == gm.items ? (gm.items + 7) / 8 * 8 : gm.main_items + ((gm.items - gm.main_items) * 2 + 7) / 8 * 8;
    if (gm.T < 1 || gm.T >= 0x7fffffffll || grid >= 0x7fffffffll || (int64_t)(cs.N * (int64_t)cs.H + 8) * cs.W * std::max(gm.red, gm.outc) * 4 >= ((int64_t)1 << 32) - 65536)
        throw KernelError("conv_winograd_fused: shape out of range (input and output must have fewer than 2^32 bytes each)");
    const int out_pad = gm.kblocks * FK;
    const int64_t fe = (int64_t)out_pad * gm.red;
    const dim3 fg((unsigned)((fe + 255) / 256)), blk(256), wg(512);
    const BnAffine bn = affine ? *affine : BnAffine{};
    const dim3 gd((unsigned)grid);
    if (adjoint) {
        hipLaunchKernelGGL(wino4_filter_fused_kernel<true>, fg, blk, 0, st, w, ws, cs.K, cs.C, out_pad);
        if (accumulate) hipLaunchKernelGGL((wino4_fused_kernel<true, 1>), gd, wg, 0, st, in, (const float *)ws, out, gm, bn);
        else hipLaunchKernelGGL((wino4_fused_kernel<true, 0>), gd, wg, 0, st, in, (const float *)ws, out, gm, bn);
    } else {
        hipLaunchKernelGGL(wino4_filter_fused_kernel<false>, fg, blk, 0, st, w, ws, cs.K, cs.C, out_pad);
        if (affine) hipLaunchKernelGGL((wino4_fused_kernel<false, 2>), gd, wg, 0, st, in, (const float *)ws, out, gm, bn);
        else if (accumulate) hipLaunchKernelGGL((wino4_fused_kernel<false, 1>), gd, wg, 0, st, in, (const float *)ws, out, gm, bn);
        else hipLaunchKernelGGL((wino4_fused_kernel<false, 0>), gd, wg, 0, st, in, (const float *)ws, out, gm, bn);
    }
    hip_check(hipGetLastError(), "fused winograd launch");
}

}  // namespace monet
