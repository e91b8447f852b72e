"""A second, independently written composition of the decoder step out of CPU
library routines (torch.nn.LSTMCell, conv1d, softmax, linear).  Used only as a
pin for the C oracle and for precision-budget estimates; never by the product.
"""
import torch
import torch.nn.functional as Fn


class TorchDecoder:
    def __init__(self, w, dims, dtype=torch.float64):
        self.d = dims
        self.dtype = dtype
        t = lambda a: torch.tensor(a, dtype=dtype)
        self.w = {k: t(v) for k, v in w.items()}
        H = dims["att_rnn_dim"]
        self.att = torch.nn.LSTMCell(dims["prenet_dim"] + dims["enc_dim"], H).to(dtype)
        self.dec = torch.nn.LSTMCell(dims["att_rnn_dim"] + dims["enc_dim"], dims["dec_rnn_dim"]).to(dtype)
        with torch.no_grad():
            for cell, p in ((self.att, "att"), (self.dec, "dec")):
                cell.weight_ih.copy_(self.w[p + "_w_ih"])
                cell.weight_hh.copy_(self.w[p + "_w_hh"])
                cell.bias_ih.copy_(self.w[p + "_b"])
                cell.bias_hh.zero_()

    def new_state(self, F):
        d, z = self.d, lambda n: torch.zeros(n, dtype=self.dtype)
        F = torch.tensor(F, dtype=self.dtype)
        L = F.shape[0]
        return dict(F=F, PM=F @ self.w["mem_w"].T, m=z(d["n_mel"]), a=z(d["enc_dim"]),
                    w_last=z(L), w_acc=z(L), h_att=z(d["att_rnn_dim"]), c_att=z(d["att_rnn_dim"]),
                    h_dec=z(d["dec_rnn_dim"]), c_dec=z(d["dec_rnn_dim"]))

    @torch.no_grad()
    def step(self, s):
        w, d = self.w, self.d
        p = Fn.relu(Fn.linear(Fn.relu(Fn.linear(s["m"], w["prenet1"])), w["prenet2"]))
        h, c = self.att(torch.cat([p, s["a"]])[None], (s["h_att"][None], s["c_att"][None]))
        s["h_att"], s["c_att"] = h[0], c[0]
        q = Fn.linear(s["h_att"], w["q_w"])
        if d["loc_in_channels"] == 2:
            u = torch.stack([s["w_last"], s["w_acc"]])[None]
        else:
            u = s["w_acc"][None, None]
        loc = Fn.conv1d(u, w["loc_conv"], padding=(d["loc_kernel"] - 1) // 2)[0].T   # [L, filters]
        pl = Fn.linear(loc, w["loc_w"])                                              # [L, att]
        e = torch.tanh(q[None] + pl + s["PM"]) @ w["v"]
        wt = torch.softmax(e, dim=0)
        s["a"] = wt @ s["F"]
        h, c = self.dec(torch.cat([s["h_att"], s["a"]])[None], (s["h_dec"][None], s["c_dec"][None]))
        s["h_dec"], s["c_dec"] = h[0], c[0]
        s["w_acc"] = s["w_acc"] + wt
        s["w_last"] = wt
        y = torch.cat([s["h_dec"], s["a"]])
        s["m"] = Fn.linear(y, w["mel_w"], w["mel_b"])
        stop = Fn.linear(y, w["stop_w"], w["stop_b"])[0]
        return s["m"].clone(), float(stop), e, wt
