// Value Model formulas (Sec. 5.2): per-task scores of many items are combined into one score
// each by a user formula with conditions.  The formula tree arrives flattened in postfix order
// and travels in the kernel arguments; one thread evaluates it for four items on a stack kept in
// LDS (one column per thread).  Bound by HBM: 4 * n_tasks bytes read and 4 written per item.
//   code (ops[i] & 255): 0 TASK (ops[i] >> 8)  1 CONST consts[i]  2 ADD  3 SUB  4 MUL  5 MIN
//   6 MAX  7 GT (1.0f / 0.0f)  8 SELECT (c != 0 ? x : y); every arithmetic step rounds once.
#pragma once
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

// Four items per thread: the decoding of an entry (scalar loads from the kernel arguments, the
// branch on its code) is shared by the four, which is what bounds the kernel for short rows.
constexpr int kVmItems = 4;

__device__ inline float vm_binary(int code, float a, float b)
{
    switch (code) {
    case 2: return __fadd_rn(a, b);
    case 3: return __fsub_rn(a, b);
    case 4: return __fmul_rn(a, b);
    case 5: return a < b ? a : b;
    case 6: return a > b ? a : b;
    default: return a > b ? 1.0f : 0.0f;
    }
}

__global__ __launch_bounds__(kVmThreads) void value_model_kernel(const float* __restrict__ scores, int64_t n,
                                                                 int32_t n_tasks, VmProgram prog,
                                                                 float* __restrict__ out)
{
    // [depth the formula reaches][kVmThreads]: sized by the launch, so that short formulas leave room for many workgroups
    extern __shared__ float4 vm_stack[];
    float4 (*s_stack)[kVmThreads] = reinterpret_cast<float4 (*)[kVmThreads]>(vm_stack);
    const int tid = threadIdx.x;
    const int64_t n_quads = (n + kVmItems - 1) / kVmItems;
    for (int64_t qd = (int64_t)blockIdx.x * kVmThreads + tid; qd < n_quads; qd += (int64_t)gridDim.x * kVmThreads) {
        const int64_t it0 = qd * kVmItems;
        // rows of the four items (the last quad repeats the last item; its extra results are not stored)
        const float* row[kVmItems];
#pragma unroll
        for (int u = 0; u < kVmItems; ++u) row[u] = scores + (it0 + u < n ? it0 + u : n - 1) * n_tasks;
        // Rows of up to eight scores are fetched once, with 16-byte loads where they line up: a
        // push per task would otherwise be a load whose 64 lanes touch 64 different lines.
        float tv[kVmItems][8];
        const bool cached = n_tasks <= 8;
        if (cached) {
            if ((n_tasks & 3) == 0 && (reinterpret_cast<uintptr_t>(scores) & 15) == 0) {
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
        auto task4 = [&](int t) {  // t is the same in every lane: the selects are scalar branches
            float4 r;
            switch (t) {
            case 0: r = make_float4(tv[0][0], tv[1][0], tv[2][0], tv[3][0]); break;
            case 1: r = make_float4(tv[0][1], tv[1][1], tv[2][1], tv[3][1]); break;
            case 2: r = make_float4(tv[0][2], tv[1][2], tv[2][2], tv[3][2]); break;
            case 3: r = make_float4(tv[0][3], tv[1][3], tv[2][3], tv[3][3]); break;
            case 4: r = make_float4(tv[0][4], tv[1][4], tv[2][4], tv[3][4]); break;
            case 5: r = make_float4(tv[0][5], tv[1][5], tv[2][5], tv[3][5]); break;
            case 6: r = make_float4(tv[0][6], tv[1][6], tv[2][6], tv[3][6]); break;
            default: r = make_float4(tv[0][7], tv[1][7], tv[2][7], tv[3][7]); break;
            }
            return r;
        };
        int top = 0;
        // the next entry is fetched (scalar loads from the kernel arguments) while this one runs
        int op = prog.ops[0];
        float cst = prog.consts[0];
        for (int i = 0; i < prog.n_ops; ++i) {
            const int code = op & 255, t = op >> 8;
            const float cv = cst;
            const int nx = i + 1 < kVmOps ? i + 1 : i;
            op = prog.ops[nx];
            cst = prog.consts[nx];
            if (code == 0) {
                s_stack[top++][tid] = cached ? task4(t) : make_float4(row[0][t], row[1][t], row[2][t], row[3][t]);
            } else if (code == 1) {
                s_stack[top++][tid] = make_float4(cv, cv, cv, cv);
            } else if (code == 8) {
                const float4 y = s_stack[--top][tid], x = s_stack[--top][tid], c = s_stack[top - 1][tid];
                s_stack[top - 1][tid] = make_float4(c.x != 0.0f ? x.x : y.x, c.y != 0.0f ? x.y : y.y,
                                                    c.z != 0.0f ? x.z : y.z, c.w != 0.0f ? x.w : y.w);
            } else {
                const float4 b = s_stack[--top][tid], a = s_stack[top - 1][tid];
                s_stack[top - 1][tid] = make_float4(vm_binary(code, a.x, b.x), vm_binary(code, a.y, b.y),
                                                    vm_binary(code, a.z, b.z), vm_binary(code, a.w, b.w));
            }
        }
        const float4 r = s_stack[0][tid];
        if (it0 + 3 < n && ((reinterpret_cast<uintptr_t>(out) & 15) == 0)) {
            *reinterpret_cast<float4*>(out + it0) = r;
        } else {
            if (it0 < n) out[it0] = r.x;
            if (it0 + 1 < n) out[it0 + 1] = r.y;
            if (it0 + 2 < n) out[it0 + 2] = r.z;
            if (it0 + 3 < n) out[it0 + 3] = r.w;
        }
    }
}

}  // namespace st
