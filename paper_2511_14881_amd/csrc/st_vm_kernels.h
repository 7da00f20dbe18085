// Value Model formulas (Sec. 5.2): per-task scores of many items are combined into one score
// each by a user formula with conditions.  The formula tree arrives flattened in postfix order
// in the kernel arguments; every workgroup copies it to LDS once (entries of a structure in the
// kernel arguments can only be read with constant indices: a loop over them would make the compiler
// copy the structure to private memory, per lane, and fetch every entry from there).  One thread
// evaluates the formula for four items; the top of its stack stays in registers, the rest lies in
// LDS (one column per thread).  Bound by HBM: 4 * n_tasks bytes read and 4 written per item.
//   code (ops[i] & 255): 0 TASK (ops[i] >> 8)  1 CONST consts[i]  2 ADD  3 SUB  4 MUL  5 MIN
//   6 MAX  7 GT (1.0f / 0.0f)  8 SELECT (c != 0 ? x : y); every arithmetic step rounds once.
#pragma once
#include <type_traits>

#include "st_device.h"

namespace st {

constexpr int kVmOps = 64;     // entries of a formula, at most
constexpr int kVmDepth = 16;   // stack depth, at most (checked on the host)
constexpr int kVmThreads = 256;

struct VmProgram {
    int32_t n_ops;
    int32_t ops[kVmOps];
    float consts[kVmOps];
};

// kVmItems items per thread, in groups of four (one float4 each): the decoding of an entry (its
// read from LDS, the branch on its code) is shared by all of them.
#ifndef ST_VM_ITEMS
#define ST_VM_ITEMS 4
#endif
constexpr int kVmItems = ST_VM_ITEMS;
constexpr int kVmQuads = kVmItems / 4;
static_assert(kVmItems % 4 == 0, "items per thread come in float4 groups");

// LDS of a launch: the stack below the register-held top (depth - 1 elements per thread, at
// least one), then the formula's entries
constexpr int vm_lds_slots(int depth) { return depth > 1 ? depth - 1 : 1; }
constexpr size_t vm_lds_bytes(int depth)
{
    return (size_t)vm_lds_slots(depth) * kVmQuads * kVmThreads * sizeof(float4) + kVmOps * sizeof(int2);
}
static_assert(vm_lds_bytes(kVmDepth) <= 160 * 1024, "the deepest formula fits the LDS of a compute unit");

__global__ __launch_bounds__(kVmThreads) void value_model_kernel(const float* __restrict__ scores, int64_t n,
                                                                 int32_t n_tasks, VmProgram prog,
                                                                 int32_t slots, float* __restrict__ out)
{
    // [slots][kVmQuads][kVmThreads]: sized by the launch from the depth the formula reaches, so that short formulas leave room for many workgroups
    extern __shared__ float4 vm_stack[];
    float4 (*s_stack)[kVmQuads][kVmThreads] = reinterpret_cast<float4 (*)[kVmQuads][kVmThreads]>(vm_stack);
    int2* s_prog = reinterpret_cast<int2*>(vm_stack + (size_t)slots * kVmQuads * kVmThreads);  // {ops[i], bits of consts[i]}
    if (threadIdx.x == 0) {
#pragma unroll
        for (int i = 0; i < kVmOps; ++i) s_prog[i] = make_int2(prog.ops[i], __float_as_int(prog.consts[i]));
    }
    __syncthreads();
    const int tid = threadIdx.x;
    const int64_t n_sets = (n + kVmItems - 1) / kVmItems;
    const bool aligned_in = (n_tasks & 3) == 0 && (reinterpret_cast<uintptr_t>(scores) & 15) == 0;
    const bool aligned_out = (reinterpret_cast<uintptr_t>(out) & 15) == 0;
    for (int64_t st = (int64_t)blockIdx.x * kVmThreads + tid; st < n_sets; st += (int64_t)gridDim.x * kVmThreads) {
        const int64_t it0 = st * kVmItems;
        // rows of the thread's items (past the end the last item is repeated; those results are not stored)
        const float* row[kVmItems];
#pragma unroll
        for (int u = 0; u < kVmItems; ++u) row[u] = scores + (it0 + u < n ? it0 + u : n - 1) * n_tasks;
        // Rows of up to eight scores are fetched once, with 16-byte loads where they line up: a
        // push per task would otherwise be a load whose 64 lanes touch 64 different lines.
        float tv[kVmItems][8];
        const bool cached = n_tasks <= 8;
        if (cached) {
            if (aligned_in) {
#pragma unroll
                for (int u = 0; u < kVmItems; ++u)
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                        if (h * 4 < n_tasks) v = reinterpret_cast<const float4*>(row[u])[h];
                        tv[u][h * 4 + 0] = v.x; tv[u][h * 4 + 1] = v.y; tv[u][h * 4 + 2] = v.z; tv[u][h * 4 + 3] = v.w;
                    }
            } else {
#pragma unroll
                for (int u = 0; u < kVmItems; ++u)
#pragma unroll
                    for (int t = 0; t < 8; ++t) tv[u][t] = t < n_tasks ? row[u][t] : 0.0f;
            }
        }
        // score t of items 4g .. 4g+3.  t is the same in every lane, so the switch is a scalar branch;
        // the (empty) assembly statement in every case keeps the compiler from folding the cases into
        // one access indexed by t, which would move the rows from registers to private memory.
        auto task4 = [&](int t, auto quad) {
            constexpr int g = decltype(quad)::value;
            float4 r;
#define VMK_CASE(k)                                                                               \
    case k:                                                                                       \
        r = make_float4(tv[4 * g][k], tv[4 * g + 1][k], tv[4 * g + 2][k], tv[4 * g + 3][k]);      \
        asm volatile("; task " #k);                                                               \
        break;
            switch (t) {
                VMK_CASE(0) VMK_CASE(1) VMK_CASE(2) VMK_CASE(3) VMK_CASE(4) VMK_CASE(5) VMK_CASE(6)
            default:
                r = make_float4(tv[4 * g][7], tv[4 * g + 1][7], tv[4 * g + 2][7], tv[4 * g + 3][7]);
                break;
            }
#undef VMK_CASE
            return r;
        };
        // Element e of the stack lies in s_stack[e] while it is not the top; the top is `tos`.
        int top = 0;  // elements on the stack (the same in every lane, like everything decoded below)
        float4 tos[kVmQuads];
#pragma unroll
        for (int g = 0; g < kVmQuads; ++g) tos[g] = make_float4(0.f, 0.f, 0.f, 0.f);
        int2 e = s_prog[0];
        for (int i = 0; i < prog.n_ops; ++i) {
            const int op = __builtin_amdgcn_readfirstlane(e.x);
            const float cv = __int_as_float(__builtin_amdgcn_readfirstlane(e.y));
            const int code = op & 255, t = op >> 8;
            e = s_prog[i + 1 < kVmOps ? i + 1 : i];  // the next entry, while this one runs
            if (code <= 1) {
                if (top > 0) {
#pragma unroll
                    for (int g = 0; g < kVmQuads; ++g) s_stack[top - 1][g][tid] = tos[g];
                }
                ++top;
                if (code == 1) {
#pragma unroll
                    for (int g = 0; g < kVmQuads; ++g) tos[g] = make_float4(cv, cv, cv, cv);
                } else if (cached) {
                    tos[0] = task4(t, std::integral_constant<int, 0>{});
                    if constexpr (kVmQuads > 1) tos[kVmQuads > 1 ? 1 : 0] = task4(t, std::integral_constant<int, (kVmQuads > 1 ? 1 : 0)>{});
                    static_assert(kVmQuads <= 2, "one fetch per quad is written out above");
                } else {
#pragma unroll
                    for (int g = 0; g < kVmQuads; ++g)
                        tos[g] = make_float4(row[4 * g][t], row[4 * g + 1][t], row[4 * g + 2][t], row[4 * g + 3][t]);
                }
            } else if (code == 8) {
#pragma unroll
                for (int g = 0; g < kVmQuads; ++g) {
                    const float4 y = tos[g], x = s_stack[top - 2][g][tid], c = s_stack[top - 3][g][tid];
                    tos[g] = make_float4(c.x != 0.0f ? x.x : y.x, c.y != 0.0f ? x.y : y.y, c.z != 0.0f ? x.z : y.z,
                                         c.w != 0.0f ? x.w : y.w);
                }
                top -= 2;
            } else {
                float4 a[kVmQuads];
#pragma unroll
                for (int g = 0; g < kVmQuads; ++g) a[g] = s_stack[top - 2][g][tid];
                --top;
#define VMK_EACH(EXPR)                                                                              \
    _Pragma("unroll") for (int g = 0; g < kVmQuads; ++g)                                              \
    {                                                                                                 \
        const float4 x = a[g], y = tos[g];                                                            \
        tos[g] = make_float4(EXPR(x.x, y.x), EXPR(x.y, y.y), EXPR(x.z, y.z), EXPR(x.w, y.w));         \
    }
#define VMK_MIN(p, q) ((p) < (q) ? (p) : (q))
#define VMK_MAX(p, q) ((p) > (q) ? (p) : (q))
#define VMK_GT(p, q) ((p) > (q) ? 1.0f : 0.0f)
                switch (code) {
                case 2: VMK_EACH(__fadd_rn) break;
                case 3: VMK_EACH(__fsub_rn) break;
                case 4: VMK_EACH(__fmul_rn) break;
                case 5: VMK_EACH(VMK_MIN) break;
                case 6: VMK_EACH(VMK_MAX) break;
                default: VMK_EACH(VMK_GT) break;
                }
#undef VMK_EACH
#undef VMK_MIN
#undef VMK_MAX
#undef VMK_GT
            }
        }
#pragma unroll
        for (int g = 0; g < kVmQuads; ++g) {
            const float4 r = tos[g];
            const int64_t i0 = it0 + 4 * g;
            if (i0 + 3 < n && aligned_out) {
                *reinterpret_cast<float4*>(out + i0) = r;
            } else {
                if (i0 < n) out[i0] = r.x;
                if (i0 + 1 < n) out[i0 + 1] = r.y;
                if (i0 + 2 < n) out[i0 + 2] = r.z;
                if (i0 + 3 < n) out[i0 + 3] = r.w;
            }
        }
    }
}

}  // namespace st
