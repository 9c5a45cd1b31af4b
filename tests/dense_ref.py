"""Independent float64 re-statement of the decoder layer with torch CPU ops, used
only to pin the oracle.  It shares nothing with the oracle: no paged cache (each
sequence keeps dense K/V history tensors), rotary embedding as a complex
multiplication, attention through ``scaled_dot_product_attention`` with an
explicit mask, library ``rms_norm`` / ``silu``."""
import torch
import torch.nn.functional as F


class DenseStage:
    def __init__(self, shape, layers_f32):
        """``layers_f32``: list of dicts name -> numpy float32 arrays."""
        self.s = shape
        self.layers = [{k: torch.from_numpy(v).double() for k, v in lw.items()} for lw in layers_f32]
        self.hist = {}      # (layer, seq) -> (K [n,Hkv,D], V [n,Hkv,D])

    def _rot(self, u, pos):
        # u [n, heads, D]; pos [n]
        D = self.s.head_dim
        inv = self.s.rope_base ** (-torch.arange(D // 2, dtype=torch.float64) * 2.0 / D)
        ang = pos.double()[:, None] * inv[None, :]
        z = torch.complex(u[..., : D // 2], u[..., D // 2:]) * torch.polar(torch.ones_like(ang), ang)[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    def forward(self, seq_ids, q_lens, ctx_lens, hidden):
        """hidden: float64 tensor [T,H], tokens packed by sequence."""
        s = self.s
        x = hidden.clone()
        rep = s.n_q_heads // s.n_kv_heads
        for li, L in enumerate(self.layers):
            n = F.rms_norm(x, (s.hidden,), L["g_attn"], eps=s.rms_eps)
            q = (n @ L["wq"].T).view(-1, s.n_q_heads, s.head_dim)
            k = (n @ L["wk"].T).view(-1, s.n_kv_heads, s.head_dim)
            v = (n @ L["wv"].T).view(-1, s.n_kv_heads, s.head_dim)
            o = torch.empty_like(q)
            at = 0
            for sid, ql, c in zip(seq_ids, q_lens, ctx_lens):
                pos = torch.arange(c, c + ql)
                qs = self._rot(q[at:at + ql], pos)
                ks = self._rot(k[at:at + ql], pos)
                Kh, Vh = self.hist.get((li, sid), (ks[:0], ks[:0]))
                assert Kh.shape[0] == c
                Kh = torch.cat([Kh, ks]); Vh = torch.cat([Vh, v[at:at + ql]])
                self.hist[(li, sid)] = (Kh, Vh)
                mask = torch.arange(c + ql)[None, :] <= pos[:, None]          # [ql, c+ql]
                o[at:at + ql] = F.scaled_dot_product_attention(
                    qs.permute(1, 0, 2), Kh.permute(1, 0, 2).repeat_interleave(rep, 0),
                    Vh.permute(1, 0, 2).repeat_interleave(rep, 0), attn_mask=mask[None]).permute(1, 0, 2)
                at += ql
            h = x + o.reshape(-1, s.n_q_heads * s.head_dim) @ L["wo"].T
            m = F.rms_norm(h, (s.hidden,), L["g_ffn"], eps=s.rms_eps)
            x = h + (F.silu(m @ L["w_gate"].T) * (m @ L["w_up"].T)) @ L["w_down"].T
        return x


class DenseOptStage:
    """The OPT-style layer (LayerNorm with bias, biased projections, no rotary embedding, ReLU
    feed-forward) re-stated with torch library ops on dense per-sequence K/V histories."""

    def __init__(self, shape, layers_f32):
        self.s = shape
        self.layers = [{k: torch.from_numpy(v).double() for k, v in lw.items()} for lw in layers_f32]
        self.hist = {}

    def forward(self, seq_ids, q_lens, ctx_lens, hidden):
        s = self.s
        x = hidden.clone()
        rep = s.n_q_heads // s.n_kv_heads
        for li, L in enumerate(self.layers):
            n = F.layer_norm(x, (s.hidden,), L["ln1_g"], L["ln1_b"], eps=s.rms_eps)
            q = F.linear(n, L["wq"], L["bq"]).view(-1, s.n_q_heads, s.head_dim)
            k = F.linear(n, L["wk"], L["bk"]).view(-1, s.n_kv_heads, s.head_dim)
            v = F.linear(n, L["wv"], L["bv"]).view(-1, s.n_kv_heads, s.head_dim)
            o = torch.empty_like(q)
            at = 0
            for sid, ql, c in zip(seq_ids, q_lens, ctx_lens):
                pos = torch.arange(c, c + ql)
                Kh, Vh = self.hist.get((li, sid), (k[:0], k[:0]))
                assert Kh.shape[0] == c
                Kh = torch.cat([Kh, k[at:at + ql]]); Vh = torch.cat([Vh, v[at:at + ql]])
                self.hist[(li, sid)] = (Kh, Vh)
                mask = torch.arange(c + ql)[None, :] <= pos[:, None]
                o[at:at + ql] = F.scaled_dot_product_attention(
                    q[at:at + ql].permute(1, 0, 2), Kh.permute(1, 0, 2).repeat_interleave(rep, 0),
                    Vh.permute(1, 0, 2).repeat_interleave(rep, 0), attn_mask=mask[None]).permute(1, 0, 2)
                at += ql
            h = x + F.linear(o.reshape(-1, s.n_q_heads * s.head_dim), L["wo"], L["bo"])
            m = F.layer_norm(h, (s.hidden,), L["ln2_g"], L["ln2_b"], eps=s.rms_eps)
            x = h + F.linear(F.relu(F.linear(m, L["w_fc1"], L["b_fc1"])), L["w_fc2"], L["b_fc2"])
        return x
