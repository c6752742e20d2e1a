"""One knowledge-distillation micro-batch step (oracle): frozen teacher section
forward, student section forward, KL loss on the two sets of logits, student
backward (paper Sec. 2.2 and Sec. 3.1)."""
from .kd import kd_loss_forward_backward
from .rounding import identity
from .section import section_backward, section_forward


def distill_step(t_spec, t_w, s_spec, s_w, cu_seqlens, ids, w_t_head, w_s_head,
                 temperature, loss_scale, rnd=identity, rnd_res=None):
    h_t = section_forward(t_spec, t_w, cu_seqlens, ids, rnd, rnd_res=rnd_res)
    h_s, cache = section_forward(s_spec, s_w, cu_seqlens, ids, rnd, keep=True, rnd_res=rnd_res)
    kd = kd_loss_forward_backward(h_t, h_s, w_t_head, w_s_head, temperature, loss_scale, rnd)
    grads, _ = section_backward(s_spec, s_w, cu_seqlens, cache, kd["d_h_s"], rnd)
    return dict(h_t=h_t, h_s=h_s, loss=kd["loss"], kl_tok=kd["kl_tok"], d_h_s=kd["d_h_s"],
                d_w_s=kd["d_w_s"], grads=grads)
