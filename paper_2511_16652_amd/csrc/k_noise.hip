// eggroll_noise_gen: materialise factor entries [member][n] from the counter-based stream
// (Sec. 1: the factors are reconstructed on demand rather than kept; Alg. 1 sampling lines).
// One thread expands one Threefry block: two normals, two raw words, or eight bounded integers.
// Integer-ALU bound; stores are contiguous per wave.
#include "common.hpp"

namespace egg {

enum NoiseMode { NM_F32 = 0, NM_BF16 = 1, NM_I8 = 2, NM_RAW = 3, NM_I8_TABLE = 4 };

template <int MODE>
__global__ __launch_bounds__(256) void noise_gen_kernel(StreamKey key, uint32_t member_begin, int64_t members,
                                                        int64_t n, int64_t blocks_per_member, IntMap im,
                                                        const int8_t* __restrict__ table, void* __restrict__ out)
{
    constexpr int VPB = (MODE == NM_I8) ? 8 : (MODE == NM_I8_TABLE ? 4 : 2);  // values per Threefry block
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= members * blocks_per_member) return;
    const int64_t m = gid / blocks_per_member;
    const uint32_t blk = (uint32_t)(gid - m * blocks_per_member);
    uint32_t w0, w1;
    noise_words(key, member_begin + (uint32_t)m, blk, w0, w1);
    const int64_t first = (int64_t)blk * VPB;  // index of this block's first value inside the member's vector
    const int64_t base = m * n + first;
    const bool full = first + VPB <= n;

    if constexpr (MODE == NM_F32 || MODE == NM_BF16) {
        float z0, z1;
        normal_pair<MODE == NM_F32>(w0, w1, z0, z1);
        if constexpr (MODE == NM_F32) {
            float* o = (float*)out + base;
            if (full && ((base & 1) == 0)) {
                *(float2*)o = make_float2(z0, z1);
            } else {
                o[0] = z0;
                if (full) o[1] = z1;
            }
        } else {
            uint16_t* o = (uint16_t*)out + base;
            const uint32_t pk = pack_bf16x2(z0, z1);
            if (full && ((base & 1) == 0)) {
                *(uint32_t*)o = pk;
            } else {
                o[0] = (uint16_t)(pk & 0xFFFFu);
                if (full) o[1] = (uint16_t)(pk >> 16);
            }
        }
    } else if constexpr (MODE == NM_RAW) {
        uint32_t* o = (uint32_t*)out + base;
        if (full && ((base & 1) == 0)) {
            *(uint2*)o = make_uint2(w0, w1);
        } else {
            o[0] = w0;
            if (full) o[1] = w1;
        }
    } else if constexpr (MODE == NM_I8_TABLE) {
        // value v of the block: 16-bit half v & 1 (low half first) of word v >> 1 indexes the table
        const uint32_t pk = (uint32_t)(uint8_t)table[w0 & 0xFFFFu] | ((uint32_t)(uint8_t)table[w0 >> 16] << 8) |
                            ((uint32_t)(uint8_t)table[w1 & 0xFFFFu] << 16) | ((uint32_t)(uint8_t)table[w1 >> 16] << 24);
        int8_t* o = (int8_t*)out + base;
        if (full && ((base & 3) == 0)) {
            *(uint32_t*)o = pk;
        } else {
            for (int b = 0; b < 4 && first + b < n; ++b) o[b] = (int8_t)((pk >> (8 * b)) & 0xFFu);
        }
    } else {
        const uint32_t p0 = int4_from_word(im, w0), p1 = int4_from_word(im, w1);
        int8_t* o = (int8_t*)out + base;
        if (full && ((base & 7) == 0)) {
            *(uint2*)o = make_uint2(p0, p1);
        } else {
            for (int b = 0; b < 8 && first + b < n; ++b) o[b] = (int8_t)(((b < 4 ? p0 : p1) >> (8 * (b & 3))) & 0xFFu);
        }
    }
}

egg_status launch_noise(eggroll_ctx* c, const StreamKey& k, uint32_t member_begin, int64_t members, int64_t n,
                        egg_dtype dtype, egg_dist dist, int int_bound, void* out)
{
    const bool table = dist == EGG_NORMAL_INT16 || (dist == EGG_UNIFORM_INT && int_bound == EGG_INT_NOISE_NORMAL16);
    const int vpb = table ? 4 : (dist == EGG_UNIFORM_INT ? 8 : 2);
    if (table && !c->norm_tab.p) {
        // first use on this context: build the table on the host and upload it (a blocking copy)
        std::vector<int8_t> h(65536);
        normal_int_table(h.data());
        egg_status st = reserve(c, c->norm_tab, 65536);
        if (st != EGG_OK) return st;
        if ((st = check_hip(c, hipMemcpy(c->norm_tab.p, h.data(), 65536, hipMemcpyHostToDevice), "upload of the integer normal table")) != EGG_OK) return st;
    }
    const int64_t bpm = (n + vpb - 1) / vpb;
    if (bpm > (int64_t(1) << 32)) return fail(c, EGG_EUNSUPPORTED, "factor vector too long");
    const int64_t total = members * bpm;
    const int64_t grid = (total + 255) / 256;
    if (grid > 0x7FFFFFFF) return fail(c, EGG_EUNSUPPORTED, "noise_gen: too many elements for one call");
    IntMap im = make_int_map(dist == EGG_UNIFORM_INT && !table ? int_bound : 0);
    const int8_t* tab = (const int8_t*)c->norm_tab.p;
    KernelScope ks(c, "noise_gen");
    const dim3 g((unsigned)grid), b(256);
    if (dist == EGG_RAW)
        hipLaunchKernelGGL(noise_gen_kernel<NM_RAW>, g, b, 0, c->stream, k, member_begin, members, n, bpm, im, tab, out);
    else if (table)
        hipLaunchKernelGGL(noise_gen_kernel<NM_I8_TABLE>, g, b, 0, c->stream, k, member_begin, members, n, bpm, im, tab, out);
    else if (dist == EGG_UNIFORM_INT)
        hipLaunchKernelGGL(noise_gen_kernel<NM_I8>, g, b, 0, c->stream, k, member_begin, members, n, bpm, im, tab, out);
    else if (dtype == EGG_F32)
        hipLaunchKernelGGL(noise_gen_kernel<NM_F32>, g, b, 0, c->stream, k, member_begin, members, n, bpm, im, tab, out);
    else
        hipLaunchKernelGGL(noise_gen_kernel<NM_BF16>, g, b, 0, c->stream, k, member_begin, members, n, bpm, im, tab, out);
    return check_hip(c, hipGetLastError(), "noise_gen launch");
}

}  // namespace egg
