// Fitting step (Eq. 1) on the fp16 matrix cores: the three contractions of a layer (forward, backward, weight
// gradient) run as v_mfma_f32_16x16x32_f16 with every fp32 operand carried as an exact-sum pair of halfs,
// hi = fp16(x), lo = fp16(x - hi), three terms per product (hi*hi + hi*lo + lo*hi, fp32 accumulate): ~22 significant
// bits per product at a third of the fp32 matrix instruction's time, and the fp16 matrix pipe runs beside the vector ALU
// that does the sines, cosines and splits.
//
// One workgroup per image, 8 wavefronts (2 at padded width 16), 16 pixels of a chunk per wavefront: a wavefront takes its
// pixels through all layers forward and backward with the activations and errors in registers (lane = (pixel n, group g);
// a 16-row tile of a layer's units is one quad of four registers per lane, rows 16 t + 4 g + v).  A quad is exactly
// half of the B operand of one 32-deep matrix step (two tiles' quads side by side), so nothing moves between lanes from
// one layer to the next, in either direction.  The weights sit in LDS once, row-major [out][in] as a hi and a lo plane:
// the forward product reads its A operand (4 consecutive inputs of one output row) with plain 8-byte reads, the backward
// product reads the transposed operand (4 consecutive output rows of one input column) with the transposing LDS read
// ds_read_b64_tr_b16 (within 16 lanes, lane i receives element i % 4 of the chunks that lanes i / 4, 4 + i / 4,
// 8 + i / 4, 12 + i / 4 point at).  Only the weight gradient, which contracts over pixels, needs other wavefronts' data:
// per layer every wavefront writes its pixels' error and layer input as hi/lo planes [pixel][unit] to LDS, and after a
// barrier each wavefront accumulates the gradient tiles it owns over the chunk's pixels, both operands read with the
// transposing read; with PL sets of planes, PL layers share one pair of barriers.  The bias is the weight of a unit of
// ones, placed right behind the layer's inputs where the padded width has room.  Gradient tiles stay in their owner's
// registers for the whole step; Adam is applied in place at the end, as in the fp32 kernel.
//
// Range of the error in fp16: the error of layer l is carried times a power of two T_l.  T of the output layer is
// chosen from the root-mean-square error the previous step saw (kept per image; 0.25 if there was none), so that the
// scaled error is around 2^4 and at most 2^15 for errors up to 4; going down, each layer multiplies by the power of two
// nearest to the inverse of its estimated gain (0.7 * sqrt(sum of squared weights / inputs), from the weights at hand),
// which keeps the scaled error's magnitude level through deep models.  The split of the error rounds toward zero, which
// saturates at the largest half instead of producing infinities; 1 / T_l goes into the factor that the accumulated
// gradient is multiplied by at the end.
#pragma once

namespace fit16 {

typedef _Float16 h4v __attribute__((ext_vector_type(4)));
typedef _Float16 h2v __attribute__((ext_vector_type(2)));
typedef short s4v __attribute__((ext_vector_type(4)));
typedef float f2v __attribute__((ext_vector_type(2)));

// Wavefronts per workgroup: 8 (128 pixels per chunk); 2 at padded width 16 (32 pixels per chunk), whose phases are so short
// that many small workgroups per CU, each at its own barrier, fill the machine better (3 x 15 at 32 x 32: 0.105 -> 0.092 ms).
constexpr int fit16_waves(int wp) { return wp == 16 ? 2 : 8; }

// Shapes and the LDS layout (bytes) for hidden widths <= WP (a multiple of 16) and L linear layers.
template <int WP, int PL = 1> struct Shape {
    static constexpr int NW = fit16_waves(WP), NTHREADS = 64 * NW, PC = 16 * NW, KS = PC / 32;   // wavefronts, threads, pixels per chunk, 32-pixel steps
    static constexpr int MT = WP / 16;            // 16-row tiles of a hidden layer
    static constexpr int NIT = MT + 1;            // column tiles of a weight gradient: the inputs, then the tile whose first column is the bias
    static constexpr int WPP = WP + 4;            // halfs per weight row (the pad spreads 16 rows over the banks)
    static constexpr int EP = WP + 4;             // halfs per pixel of the error planes
    static constexpr int HP = WP + 20;            // halfs per pixel of the input planes: WP units, the unit of ones, 15 zero units, pad
    static constexpr int GSLOTS = (MT * NIT + NW - 1) / NW;   // gradient tiles a wavefront owns per layer
    // LDS, in this order: the sets of pixel planes, the first layer, the biases (12 slots), the hidden layers' weight planes,
    // the output layer's, a pad, small tables.  Everything up to the hidden layers sits at compile-time offsets, so a lane's
    // address is one register plus an immediate.  Reads that run past an operand's rows or columns (the other half of an
    // odd last tile, whose partner operand is zero) land in what follows: weight planes, then the pad of zeros.
    static constexpr uint32_t SET = 4u * PC * (EP + HP);                                                // bytes of one set of planes (error hi, lo; input hi, lo)
    static __host__ __device__ constexpr uint32_t off_eh(int j) { return (uint32_t)j * SET; }
    static __host__ __device__ constexpr uint32_t off_el(int j) { return off_eh(j) + 2u * PC * EP; }
    static __host__ __device__ constexpr uint32_t off_hh(int j) { return off_el(j) + 2u * PC * EP; }
    static __host__ __device__ constexpr uint32_t off_hl(int j) { return off_hh(j) + 2u * PC * HP; }
    static __host__ __device__ constexpr uint32_t off_w0() { return PL * SET; }                           // float [WP][4]: x weight, y weight, bias, 0
    static __host__ __device__ constexpr uint32_t off_bias(int l) { return off_w0() + WP * 16 + (uint32_t)l * WP * 4; }   // float [WP] per layer
    static __host__ __device__ constexpr uint32_t off_hid(int l) { return off_bias(12) + (uint32_t)(l - 1) * 4u * WP * WPP; }   // hi plane, then lo plane
    static __host__ __device__ constexpr uint32_t off_last(int L) { return off_hid(L - 1); }              // [16][WPP] hi, then lo
    static constexpr uint32_t PAD = (2u * 16 * WPP + 15) / 16 * 16 + 64;
    static __host__ __device__ constexpr uint32_t off_misc(int L) { return off_last(L) + 4u * 16 * WPP + PAD; }   // float [16 + 16 + 16 * 8]: factors, scales, partial sums
    static __host__ __device__ constexpr uint32_t total(int L) { return off_misc(L) + 4u * (32 + 16 * 8); }
};

typedef _Float16 h8v __attribute__((ext_vector_type(8)));
// One matrix step is v_mfma_f32_16x16x32_f16 (the 16-deep instruction runs at half its rate on this chip): lane group g
// supplies k = 8 g .. 8 g + 7, taken as the quads of two tiles (k = 4 g + v of tile 2 j, then of tile 2 j + 1); both
// operands of a product are built the same way, so the order within the 32 is immaterial.  An odd last tile pairs with zeros.
__device__ __forceinline__ h8v cat(h4v a, h4v b) { return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7); }
__device__ __forceinline__ f32x4 mfma32(h8v a, h8v b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0); }
// a x b with both operands as hi/lo pairs
__device__ __forceinline__ f32x4 mfma3(h8v ah, h8v al, h8v bh, h8v bl, f32x4 c) {
    c = mfma32(ah, bh, c);
    c = mfma32(ah, bl, c);
    return mfma32(al, bh, c);
}
// transposing LDS read: see the file header; p is this lane's chunk of 4 halfs
__device__ __forceinline__ h4v read_tr(const char *p) {
    const s4v v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s4v *)p);
    return __builtin_bit_cast(h4v, v);
}
// exact hi/lo split of a quad, round to nearest (activations, |x| <= 1).  neg1 is -1.0f passed as data, so that
// x - float(hi) stays one mixed-precision fma instead of a conversion and a subtraction.
__device__ __forceinline__ void split_rne(f32x4 x, float neg1, h4v &hi, h4v &lo) {
    const f2v p0 = {x[0], x[1]}, p1 = {x[2], x[3]};
    const h2v a0 = __builtin_convertvector(p0, h2v), a1 = __builtin_convertvector(p1, h2v);
    const f2v r0 = {__builtin_fmaf((float)a0[0], neg1, x[0]), __builtin_fmaf((float)a0[1], neg1, x[1])};
    const f2v r1 = {__builtin_fmaf((float)a1[0], neg1, x[2]), __builtin_fmaf((float)a1[1], neg1, x[3])};
    const h2v b0 = __builtin_convertvector(r0, h2v), b1 = __builtin_convertvector(r1, h2v);
    hi = (h4v){a0[0], a0[1], a1[0], a1[1]};
    lo = (h4v){b0[0], b0[1], b1[0], b1[1]};
}
// hi/lo split of a quad, round toward zero: values beyond the largest half saturate there instead of becoming infinite
__device__ __forceinline__ void split_rtz(f32x4 x, float neg1, h4v &hi, h4v &lo) {
    const auto a0 = __builtin_amdgcn_cvt_pkrtz(x[0], x[1]), a1 = __builtin_amdgcn_cvt_pkrtz(x[2], x[3]);
    const auto b0 = __builtin_amdgcn_cvt_pkrtz(__builtin_fmaf((float)a0[0], neg1, x[0]), __builtin_fmaf((float)a0[1], neg1, x[1]));
    const auto b1 = __builtin_amdgcn_cvt_pkrtz(__builtin_fmaf((float)a1[0], neg1, x[2]), __builtin_fmaf((float)a1[1], neg1, x[3]));
    hi = (h4v){(_Float16)a0[0], (_Float16)a0[1], (_Float16)a1[0], (_Float16)a1[1]};
    lo = (h4v){(_Float16)b0[0], (_Float16)b0[1], (_Float16)b1[0], (_Float16)b1[1]};
}
__device__ __forceinline__ f32x4 sin4(f32x4 z) {
    return (f32x4){__builtin_amdgcn_sinf(z[0]), __builtin_amdgcn_sinf(z[1]), __builtin_amdgcn_sinf(z[2]), __builtin_amdgcn_sinf(z[3])};
}

// The unit of ones (its weight is the bias): right behind a layer's inputs where the padded width has room, else at WP.
template <int WP> __device__ __forceinline__ int ones_unit(int din) { return din < WP ? din : WP; }
// Where entry (row o, input unit j) of layer l's gradient lives in the parameter vector, or -1 (padding).
template <int WP> __device__ __forceinline__ int param_index(const FitArgs &a, int l, int o, int j) {
    const int din = a.d[l], dout = a.d[l + 1];
    if (o >= dout) return -1;
    if (j == ones_unit<WP>(din)) return a.p_off[l] + dout * din + o;
    return j < din ? a.p_off[l] + o * din + j : -1;
}

template <int WP, int ML, int PL>
__global__ __launch_bounds__(Shape<WP>::NTHREADS, (Shape<WP>::NW <= 4 && ML <= 4) ? 4 : 2) void fit16_step_kernel(const FitArgs a) {
    typedef Shape<WP, PL> S;
    constexpr int kWaves = S::NW, kThreads = S::NTHREADS, kPC = S::PC;
    constexpr int MT = S::MT, NP = (MT + 1) / 2, WPP = S::WPP, EP = S::EP, HP = S::HP, GSLOTS = S::GSLOTS;
    const h4v zh = {(_Float16)0.0f, (_Float16)0.0f, (_Float16)0.0f, (_Float16)0.0f};
    extern __shared__ __attribute__((aligned(16))) char lds16[];
    char *const lds = lds16;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, n = lane & 15, g = lane >> 4;
    const size_t img = blockIdx.x;
    float *P = a.params + img * a.n_params;
    const f32x4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    const float neg1 = a.neg1;
    const int L0 = a.L;
    float *const misc = (float *)(lds + S::off_misc(L0));      // [0..15] gradient factor per layer, [16..31] scale r per layer, [32..] partial sums
    char *const EH0 = lds + S::off_eh(0), *const EL0 = lds + S::off_el(0), *const HH0 = lds + S::off_hh(0), *const HL0 = lds + S::off_hl(0);   // set 0; set j is j * S::SET further

    // ---- set up: zero everything; weights as hi/lo planes (sine layers times w0 / 2pi: Z comes out in revolutions), biases,
    //      the unit of ones; per layer the sum of squared weights (for the error's scale), summed in a fixed order
    for (uint32_t q = tid; q < S::total(L0) / 16; q += kThreads) ((uint4 *)lds)[q] = make_uint4(0u, 0u, 0u, 0u);
    __syncthreads();
    for (int l = 0; l < L0; ++l) {
        const int din = a.d[l], dout = a.d[l + 1];
        const float *src = P + a.p_off[l];
        const float sc = l < L0 - 1 ? a.w0rev : 1.0f;
        float ss = 0.0f;
        if (l == 0) {
            float *W0 = (float *)(lds + S::off_w0());
            for (int e = tid; e < dout * 2; e += kThreads) { const float w = src[e] * sc; W0[(e >> 1) * 4 + (e & 1)] = w; }
            for (int o = tid; o < dout; o += kThreads) W0[o * 4 + 2] = src[dout * din + o] * sc;
        } else {
            _Float16 *Wh = (_Float16 *)(lds + (l == L0 - 1 ? S::off_last(L0) : S::off_hid(l)));
            _Float16 *Wl = Wh + (l == L0 - 1 ? 16 : WP) * WPP;
            float *B = (float *)(lds + S::off_bias(l));
            for (int e = tid; e < dout * din; e += kThreads) {
                const int o = e / din, i = e - o * din;
                const float w = src[e] * sc;
                const _Float16 h = (_Float16)w;
                Wh[o * WPP + i] = h;
                Wl[o * WPP + i] = (_Float16)(w - (float)h);
                ss = fmaf(w, w, ss);
            }
            for (int o = tid; o < dout; o += kThreads) B[o] = src[dout * din + o] * sc;
        }
        for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
        if (lane == 0) misc[32 + l * 8 + wave] = ss;
    }
    for (int p = tid; p < kPC * PL; p += kThreads) ((_Float16 *)(HH0 + (p / kPC) * S::SET))[(p % kPC) * HP + WP] = (_Float16)1.0f;
    __syncthreads();
    if (tid == 0) {
        // scale of the output layer's error from the error the previous step saw; then down the layers by the estimated gains
        float rms = a.emag ? a.emag[img] : 0.0f;
        rms = rms > 0.0f ? fminf(fmaxf(rms, 0.001953125f), 4.0f) : 0.25f;
        const float raw = 2.0f * a.loss_scale * rms;                        // error of the output layer before scaling, typical size
        float T = exp2f(4.0f - ceilf(log2f(raw)));
        T = fminf(fmaxf(T, 1e-30f), 1e30f);
        misc[16 + L0 - 1] = T * 2.0f * a.loss_scale;                        // what the output difference is multiplied by
        misc[L0 - 1] = a.gscale[L0 - 1] / T;
        for (int l = L0 - 1; l >= 1; --l) {
            float ss = 0.0f;
            for (int w = 0; w < kWaves; ++w) ss += misc[32 + l * 8 + w];
            const float gain = 0.7f * sqrtf(ss / (float)a.d[l]);
            float r = gain > 0.0f ? exp2f(rintf(-log2f(gain))) : 1.0f;
            r = fminf(fmaxf(r, 0.015625f), 256.0f);
            if (!(T * r < 1e30f && T * r > 1e-30f)) r = 1.0f;
            T *= r;
            misc[16 + l - 1] = r;                                           // E_{l-1} = (W_l^T E_l) cos(.) r
            misc[l - 1] = a.gscale[l - 1] / T;
        }
    }
    __syncthreads();

    f32x4 acc[ML][GSLOTS];          // weight-gradient tiles, whole step
    f32x4 zst[ML - 1][MT];          // pre-activations (revolutions) of this wavefront's 16 pixels, sine layers
#pragma unroll
    for (int l = 0; l < ML; ++l)
#pragma unroll
        for (int s = 0; s < GSLOTS; ++s) acc[l][s] = zero4;
#pragma unroll
    for (int l = 0; l < ML - 1; ++l)
#pragma unroll
        for (int t = 0; t < MT; ++t) zst[l][t] = zero4;
    float loss_part = 0.0f;

    const int pc = wave * 16 + n;                                  // this lane's pixel within the chunk
    const uint32_t nchunks = (a.HW + kPC - 1) / kPC;
    for (uint32_t c = 0; c < nchunks; ++c) {
        int L = a.L;
        asm volatile("" : "+s"(L));       // read afresh per chunk: keeps the unrolled layers' conditions out of long-lived lane masks
        uint32_t p = c * kPC + (uint32_t)pc;
        const bool valid = p < a.HW;
        p = valid ? p : a.HW - 1;
        const uint32_t row = p / a.W, col = p - row * a.W;
        const float x = fmaf(a.span, (float)(2 * col + 1) * a.inv2W, a.lo), y = fmaf(a.span, (float)(2 * row + 1) * a.inv2H, a.lo);

        // ---- forward.  Layer 0 on the vector ALU (two inputs); hidden layers: Z = W H + b, tile by tile
        h4v Bh[MT], Bl[MT];
        {
            const float4 *W0 = (const float4 *)(lds + S::off_w0());
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                f32x4 z;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float4 w = W0[16 * t + 4 * g + v];
                    z[v] = fmaf(w.x, x, fmaf(w.y, y, w.z));
                }
                zst[0][t] = z;
                split_rne(sin4(z), neg1, Bh[t], Bl[t]);
            }
        }
#pragma unroll
        for (int l = 1; l < ML - 1; ++l) {
            if (l < L - 1) {
                const char *Wh = lds + S::off_hid(l), *Wl = Wh + 2 * WP * WPP;
                const f32x4 *B = (const f32x4 *)(lds + S::off_bias(l));
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    f32x4 z = B[4 * mt + g];
#pragma unroll
                    for (int j = 0; j < NP; ++j) {
                        const int at = 2 * ((16 * mt + n) * WPP + 32 * j + 4 * g);
                        const bool two = 2 * j + 1 < MT;      // an odd last tile: the B operand's other half is zero, the A operand's is whatever follows in LDS (finite halfs)
                        const h8v ah = cat(*(const h4v *)(Wh + at), *(const h4v *)(Wh + at + 32)), al = cat(*(const h4v *)(Wl + at), *(const h4v *)(Wl + at + 32));
                        z = mfma3(ah, al, cat(Bh[2 * j], two ? Bh[2 * j + 1] : zh), cat(Bl[2 * j], two ? Bl[2 * j + 1] : zh), z);
                    }
                    zst[l][mt] = z;
                }
#pragma unroll
                for (int t = 0; t < MT; ++t) split_rne(sin4(zst[l][t]), neg1, Bh[t], Bl[t]);
            }
        }
        f32x4 E[MT];                       // the error at hand, scaled (see the file header); the output layer's is tile 0
#pragma unroll
        for (int t = 0; t < MT; ++t) E[t] = zero4;
        {
            const char *Wh = lds + S::off_last(L), *Wl = Wh + 2 * 16 * WPP;
            f32x4 z = ((const f32x4 *)(lds + S::off_bias(L - 1)))[g];
#pragma unroll
            for (int j = 0; j < NP; ++j) {
                const int at = 2 * (n * WPP + 32 * j + 4 * g);
                const bool two = 2 * j + 1 < MT;
                const h8v ah = cat(*(const h4v *)(Wh + at), *(const h4v *)(Wh + at + 32)), al = cat(*(const h4v *)(Wl + at), *(const h4v *)(Wl + at + 32));
                z = mfma3(ah, al, cat(Bh[2 * j], two ? Bh[2 * j + 1] : zh), cat(Bl[2 * j], two ? Bl[2 * j + 1] : zh), z);
            }
            const float eo = misc[16 + L - 1];
#pragma unroll
            for (int v = 0; v < 3; ++v) {
                float e = 0.0f;
                if (g == 0 && valid) e = z[v] - a.target[(img * 3 + v) * a.HW + p];
                loss_part = fmaf(e, e, loss_part);
                E[0][v] = e * eo;
            }
        }

        // ---- backward, PL layers at a time: each wavefront writes its pixels' error and layer input of those layers to LDS
        //      as hi/lo planes (one set per layer) and takes the error down through them in registers; after a barrier the
        //      weight-gradient tiles of those layers take the chunk's pixels, spread round-robin over the wavefronts
#pragma unroll
        for (int lg = ML - 1; lg >= 0; lg -= PL) {
            const int llow = lg - PL + 1 > 0 ? lg - PL + 1 : 0;
            if (llow < L) {
#pragma unroll
                for (int j = 0; j < PL; ++j) {
                    const int l = lg - j;
                    if (l >= 0 && l < L) {
                        const bool last = l == L - 1;
                        char *const EH = EH0 + j * S::SET, *const EL = EL0 + j * S::SET, *const HH = HH0 + j * S::SET, *const HL = HL0 + j * S::SET;
                        h4v Eh[MT], El[MT];
#pragma unroll
                        for (int t = 0; t < MT; ++t) {
                            split_rtz(E[t], neg1, Eh[t], El[t]);            // (the output layer's error has one tile; the others are zero)
                            if (t == 0 || !last) {
                                const int at = 2 * (pc * EP + 16 * t + 4 * g);
                                *(h4v *)(EH + at) = Eh[t];
                                *(h4v *)(EL + at) = El[t];
                            }
                        }
                        const int uo = ones_unit<WP>(a.d[l]);          // < WP: the unit of ones sits inside a tile and is written with it
                        if (l == 0) {
                            if (g == 0) {
                                h4v hi, lo;
                                split_rne((f32x4){x, y, 1.0f, 0.0f}, neg1, hi, lo);
                                *(h4v *)(HH + 2 * (pc * HP)) = hi;
                                *(h4v *)(HL + 2 * (pc * HP)) = lo;
                            }
                        } else {
                            // E_{l-1} = (W_l^T E_l) cos(2 pi z_{l-1}) r: the transposed operand straight from the row-major planes
                            const char *Wh = lds + (last ? S::off_last(L) : S::off_hid(l)), *Wl = Wh + 2 * (last ? 16 : WP) * WPP;
                            const float r = misc[16 + l - 1];
                            const int e4 = n >> 2, q4 = n & 3;
                            f32x4 gacc[MT];
#pragma unroll
                            for (int it = 0; it < MT; ++it) {
                                gacc[it] = zero4;
#pragma unroll
                                for (int jp = 0; jp < NP; ++jp) {
                                    if (jp == 0 || !last) {
                                        const int at = 2 * ((32 * jp + 4 * g + e4) * WPP + 16 * it + 4 * q4);
                                        const bool two = 2 * jp + 1 < MT;     // rows past the layer's own: whatever follows in LDS, times an error of zero
                                        const h8v ah = cat(read_tr(Wh + at), read_tr(Wh + at + 32 * WPP)), al = cat(read_tr(Wl + at), read_tr(Wl + at + 32 * WPP));
                                        gacc[it] = mfma3(ah, al, cat(Eh[2 * jp], two ? Eh[2 * jp + 1] : zh), cat(El[2 * jp], two ? El[2 * jp + 1] : zh), gacc[it]);
                                    }
                                }
                            }
                            // the layer's input again (sine of the kept pre-activations) for the weight gradient, while the matrix steps run
#pragma unroll
                            for (int t = 0; t < MT; ++t) {
                                h4v hi, lo;
                                split_rne(sin4(zst[l - 1][t]), neg1, hi, lo);
                                const int at = 2 * (pc * HP + 16 * t + 4 * g);
                                *(h4v *)(HH + at) = hi;
                                *(h4v *)(HL + at) = lo;
                            }
                            // the unit of ones inside a tile: the padded unit there was written as 0 by the lane that owns it; that lane
                            // makes it 1 (same lane, later store: program order)
                            if (uo < WP && 4 * g == (uo & 12)) ((_Float16 *)HH)[pc * HP + uo] = (_Float16)1.0f;
#pragma unroll
                            for (int it = 0; it < MT; ++it) {
                                const f32x4 z = zst[l - 1][it];
                                const f32x4 c = {__builtin_amdgcn_cosf(z[0]), __builtin_amdgcn_cosf(z[1]), __builtin_amdgcn_cosf(z[2]), __builtin_amdgcn_cosf(z[3])};
                                E[it] = gacc[it] * (c * r);
                            }
                        }
                    }
                }
                __syncthreads();
                int rot = 0;
#pragma unroll
                for (int j = 0; j < PL; ++j) {
                    const int l = lg - j;
                    if (l >= 0 && l < L) {
                        // dW_l += E_l H_l^T over the chunk's pixels: tile (rows ot, columns it), 32 pixels per matrix step
                        {
                            const bool last = l == L - 1;
                            const int uo = ones_unit<WP>(a.d[l]);
                            const char *const EH = EH0 + j * S::SET, *const EL = EL0 + j * S::SET, *const HH = HH0 + j * S::SET, *const HL = HL0 + j * S::SET;
                            int nit = uo / 16 + 1;                           // column tiles up to the one with the unit of ones
                            asm volatile("" : "+s"(nit));                  // a scalar, derived again per chunk: not a set of per-layer values held across the loop
                            const int ntasks = (last ? 1 : MT) * nit;
                            const int e4 = n >> 2, q4 = n & 3;
                            // the group's layers start their round-robin over the wavefronts where the layer before stopped
                            const int wv = (wave + kWaves - rot % kWaves) % kWaves;
                            rot += ntasks;
#pragma unroll
                            for (int s = 0; s < GSLOTS; ++s) {
                                const int task = wv + s * kWaves;
                                if (task < ntasks) {
                                    int ot = 0;
#pragma unroll
                                    for (int q = 1; q < MT; ++q) ot += task >= q * nit ? 1 : 0;
                                    const int it = task - ot * nit;
                                    f32x4 d0 = zero4, d1 = zero4, d2 = zero4;        // one chain per term: the matrix steps of a tile do not wait for each other
#pragma unroll
                                    for (int k = 0; k < kPC / 32; ++k) {
                                        const int px = 32 * k + 4 * g + e4;
                                        const int ea = 2 * (px * EP + 16 * ot + 4 * q4), ha = 2 * (px * HP + 16 * it + 4 * q4);
                                        const h8v eh = cat(read_tr(EH + ea), read_tr(EH + ea + 32 * EP)), el = cat(read_tr(EL + ea), read_tr(EL + ea + 32 * EP));
                                        const h8v hh = cat(read_tr(HH + ha), read_tr(HH + ha + 32 * HP)), hl = cat(read_tr(HL + ha), read_tr(HL + ha + 32 * HP));
                                        d0 = mfma32(eh, hh, d0);
                                        d1 = mfma32(eh, hl, d1);
                                        d2 = mfma32(el, hh, d2);
                                    }
                                    const f32x4 d = acc[l][s] + (d0 + (d1 + d2));
                                    acc[l][s] = d;
                                }
                            }
                        }
                    }
                }
                __syncthreads();
            }
        }
    }
    const int L = a.L;

    // ---- loss of this step's parameters, and the error's size for the next step's scale
    __shared__ float red[8];
    for (int off = 32; off > 0; off >>= 1) loss_part += __shfl_xor(loss_part, off, 64);
    if (lane == 0) red[wave] = loss_part;
    __syncthreads();
    if (tid == 0) {
        float s = 0.0f;
        for (int w = 0; w < kWaves; ++w) s += red[w];
        a.loss[img] = a.loss_scale * s;
        if (a.emag && !a.grad_out) a.emag[img] = sqrtf(s / (3.0f * (float)a.HW));
    }

    // ---- every gradient entry is in exactly one lane: Adam in place (or hand the gradient out)
    float *M = a.m + img * a.n_params, *V = a.v + img * a.n_params;
    const uint8_t *K = a.keep ? a.keep + img * a.n_params : nullptr;
    float *G = a.grad_out ? a.grad_out + img * a.n_params : nullptr;
#pragma unroll
    for (int lg = ML - 1; lg >= 0; lg -= PL) {
        int rot = 0;
#pragma unroll
        for (int j = 0; j < PL; ++j) {
            const int l = lg - j;
            if (l >= 0 && l < L) {
                const int nit = ones_unit<WP>(a.d[l]) / 16 + 1, ntasks = (l == L - 1 ? 1 : MT) * nit;
                const int wv = (wave + kWaves - rot % kWaves) % kWaves;        // the same owner as in the loop above
                rot += ntasks;
                const float gs = misc[l];
#pragma unroll
                for (int s = 0; s < GSLOTS; ++s) {
                    const int task = wv + s * kWaves;
                    if (task < ntasks) {
                        int ot = 0;
#pragma unroll
                        for (int q = 1; q < MT; ++q) ot += task >= q * nit ? 1 : 0;
                        const int it = task - ot * nit;
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int at = param_index<WP>(a, l, ot * 16 + 4 * g + v, it * 16 + n);
                            if (at >= 0) {
                                const bool kept = !K || K[at];
                                const float gr = kept ? acc[l][s][v] * gs : 0.0f;
                                if (G) {
                                    G[at] = gr;
                                } else if (kept) {
                                    const float mm = a.b1 * M[at] + (1.0f - a.b1) * gr;
                                    const float vv = a.b2 * V[at] + (1.0f - a.b2) * gr * gr;
                                    M[at] = mm;
                                    V[at] = vv;
                                    P[at] -= a.lr * (mm * a.c1inv) / (sqrtf(vv * a.c2inv) + a.eps);
                                } else {
                                    P[at] = 0.0f;
                                }
                            }
                        }
                    }
                }
            }
        }
    }
}

}  // namespace fit16
