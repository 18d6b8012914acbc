// Autograd wiring of the drop-in layers in C++ (Introduction, Listing 1; Algorithm 1), as torch
// operators invact::act, invact::act_pbit and invact::glu.  It does what nn.py's Python
// autograd.Function classes do -- allocate the outputs, call the C ABI of libinvact on the
// current stream, save (output, mask) for the backward -- without the interpreter on the path:
// on an MI355X the two kernels of a 2^25-element layer take about 60 us, less than two
// Python autograd.Function hops cost.  No arithmetic happens here.
//
// Built by build.py into libinvact_torch.so (host code only; links libinvact.so and libtorch).
#include <cstdint>

#include <ATen/ATen.h>
#include <c10/core/DeviceGuard.h>
#include <c10/hip/HIPStream.h>
#include <torch/csrc/autograd/custom_function.h>
#include <torch/library.h>

#include "../../include/invact.h"

namespace {

using torch::autograd::AutogradContext;
using torch::autograd::variable_list;

void check(int status)
{
    TORCH_CHECK(status == INVACT_OK, "libinvact: ", invact_strerror(status), " (status ", status, ")");
}

int dtype_of(const at::Tensor& t)
{
    TORCH_CHECK(t.is_cuda(), "InvAct layers need GPU tensors (there is no CPU path)");
    if (t.scalar_type() == at::kFloat) return INVACT_FP32;
    if (t.scalar_type() == at::kBFloat16) return INVACT_BF16;
    TORCH_CHECK(false, "InvAct layers support float32 and bfloat16, got ", t.scalar_type());
}

hipStream_t stream_of(const at::Tensor& t) { return c10::hip::getCurrentHIPStream(t.device().index()).stream(); }

// t as the library wants it: contiguous, and starting on a 16-byte boundary.  A contiguous view into the middle
// of another tensor (t.view(-1)[3:]) is contiguous but need not be aligned: it is copied.
at::Tensor dense(const at::Tensor& t)
{
    at::Tensor c = t.contiguous();
    return reinterpret_cast<uintptr_t>(c.data_ptr()) % 16 == 0 ? c : c.clone();
}

at::Tensor new_mask(const at::Tensor& like)
{
    return at::empty({(int64_t)invact_mask_bytes((size_t)like.numel())}, like.options().dtype(at::kByte));
}

struct Act : torch::autograd::Function<Act> {
    static at::Tensor forward(AutogradContext* ctx, const at::Tensor& x, int64_t kind)
    {
        const int dt = dtype_of(x);
        const at::Tensor xc = dense(x);
        at::Tensor y = at::empty_like(xc), mask = new_mask(xc);
        const c10::DeviceGuard guard(xc.device());
        check(invact_fwd((int)kind, dt, xc.data_ptr(), y.data_ptr(), mask.data_ptr(), (size_t)xc.numel(), stream_of(xc)));
        ctx->saved_data["kind"] = kind;
        ctx->save_for_backward({y, mask});
        return y;
    }
    static variable_list backward(AutogradContext* ctx, variable_list grads)
    {
        const auto saved = ctx->get_saved_variables();
        const at::Tensor &y = saved[0], &mask = saved[1];
        const at::Tensor g = dense(grads[0]);
        at::Tensor gx = at::empty_like(g);
        const c10::DeviceGuard guard(g.device());
        check(invact_bwd((int)ctx->saved_data["kind"].toInt(), dtype_of(g), y.data_ptr(), mask.data_ptr(), g.data_ptr(),
                         gx.data_ptr(), (size_t)g.numel(), stream_of(g)));
        return {gx, at::Tensor()};
    }
};

struct ActPbit : torch::autograd::Function<ActPbit> {
    static at::Tensor forward(AutogradContext* ctx, const at::Tensor& x, int64_t kind)
    {
        const int dt = dtype_of(x);
        const at::Tensor xc = dense(x);
        at::Tensor y = at::empty_like(xc);
        const c10::DeviceGuard guard(xc.device());
        check(invact_pbit_fwd((int)kind, dt, xc.data_ptr(), y.data_ptr(), (size_t)xc.numel(), stream_of(xc)));
        ctx->saved_data["kind"] = kind;
        ctx->save_for_backward({y});
        return y;
    }
    static variable_list backward(AutogradContext* ctx, variable_list grads)
    {
        const at::Tensor y = ctx->get_saved_variables()[0];
        const at::Tensor g = dense(grads[0]);
        at::Tensor gx = at::empty_like(g);
        const c10::DeviceGuard guard(g.device());
        check(invact_pbit_bwd((int)ctx->saved_data["kind"].toInt(), dtype_of(g), y.data_ptr(), g.data_ptr(), gx.data_ptr(),
                              (size_t)g.numel(), stream_of(g)));
        return {gx, at::Tensor()};
    }
};

struct Glu : torch::autograd::Function<Glu> {
    static at::Tensor forward(AutogradContext* ctx, const at::Tensor& gate, const at::Tensor& up, int64_t kind)
    {
        TORCH_CHECK(gate.sizes() == up.sizes() && gate.scalar_type() == up.scalar_type() && gate.device() == up.device(),
                    "gate and up must share shape, dtype and device");
        const int dt = dtype_of(gate);
        const at::Tensor gc = dense(gate), uc = dense(up);
        at::Tensor act = at::empty_like(gc), h = at::empty_like(gc), mask = new_mask(gc);
        const c10::DeviceGuard guard(gc.device());
        check(geglu_invact_fwd((int)kind, dt, gc.data_ptr(), uc.data_ptr(), act.data_ptr(), h.data_ptr(),
                               mask.data_ptr(), (size_t)gc.numel(), stream_of(gc)));
        ctx->saved_data["kind"] = kind;
        ctx->save_for_backward({act, uc, mask});
        return h;
    }
    static variable_list backward(AutogradContext* ctx, variable_list grads)
    {
        const auto saved = ctx->get_saved_variables();
        const at::Tensor &act = saved[0], &up = saved[1], &mask = saved[2];
        const at::Tensor g = dense(grads[0]);
        at::Tensor gg = at::empty_like(g), gu = at::empty_like(g);
        const c10::DeviceGuard guard(g.device());
        check(geglu_invact_bwd((int)ctx->saved_data["kind"].toInt(), dtype_of(g), act.data_ptr(), up.data_ptr(),
                               mask.data_ptr(), g.data_ptr(), gg.data_ptr(), gu.data_ptr(), (size_t)g.numel(), stream_of(g)));
        return {gg, gu, at::Tensor()};
    }
};

at::Tensor act(const at::Tensor& x, int64_t kind) { return Act::apply(x, kind); }
at::Tensor act_pbit(const at::Tensor& x, int64_t kind) { return ActPbit::apply(x, kind); }
at::Tensor glu(const at::Tensor& gate, const at::Tensor& up, int64_t kind) { return Glu::apply(gate, up, kind); }

}  // namespace

TORCH_LIBRARY(invact, m)
{
    m.def("act(Tensor x, int kind) -> Tensor", &act);
    m.def("act_pbit(Tensor x, int kind) -> Tensor", &act_pbit);
    m.def("glu(Tensor gate, Tensor up, int kind) -> Tensor", &glu);
}
