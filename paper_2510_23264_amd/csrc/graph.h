// Node / edge numbering of the computational graph (host side).
// Paper, Appendix "Preliminaries", Circuit Discovery: nodes are attention heads
// and MLP layers plus embedding and unembedding; a node reads the sum of its
// predecessors.  Head inputs are split into query / key / value receivers.
#pragma once
#include <stdint.h>

namespace pahq {

struct GraphDims {
  int L, H, mu, Ns, Nr;
  int C;      // inputs per head: 3 (separate query, key and value receivers) or 1 (one receiver all three projections read)
  GraphDims() : L(0), H(0), mu(0), Ns(0), Nr(0), C(3) {}
  GraphDims(int L_, int H_, bool mlp, bool split_qkv = true) : L(L_), H(H_), mu(mlp ? 1 : 0), C(split_qkv ? 3 : 1) {
    Ns = 1 + L * (H + mu);
    Nr = L * (C * H + mu) + 1;
  }
  int head(int l, int h) const { return 1 + l * (H + mu) + h; }
  int mlp(int l) const { return 1 + l * (H + mu) + H; }
  int headin(int l, int h, int c) const { return l * (C * H + mu) + C * h + (C == 3 ? c : 0); }
  int mlpin(int l) const { return l * (C * H + mu) + C * H; }
  int out() const { return Nr - 1; }
  // kind: 0 headin, 1 mlpin, 2 out; c = -1 for the single input of an unsplit head
  void receiver_info(int r, int& kind, int& l, int& h, int& c) const {
    if (r == Nr - 1) { kind = 2; l = L; h = c = -1; return; }
    l = r / (C * H + mu);
    int q = r % (C * H + mu);
    if (q < C * H) { kind = 0; h = q / C; c = C == 3 ? q % 3 : -1; } else { kind = 1; h = c = -1; }
  }
  // position on the residual stream: 2l before attention of layer l, 2l+1 before its MLP, 2L at the end
  int pos_of_receiver(int r) const {
    int k, l, h, c;
    receiver_info(r, k, l, h, c);
    return k == 0 ? 2 * l : (k == 1 ? 2 * l + 1 : 2 * L);
  }
  // number of senders upstream of a position (they are the senders 0 .. n-1)
  int n_static(int pos) const {
    if (pos >= 2 * L) return Ns;
    int l = pos / 2;
    return 1 + l * (H + mu) + ((pos & 1) ? H : 0);
  }
  int n_upstream(int r) const { return n_static(pos_of_receiver(r)); }
  int node_of_receiver(int r) const {
    int k, l, h, c;
    receiver_info(r, k, l, h, c);
    return k == 0 ? head(l, h) : (k == 1 ? mlp(l) : -1);
  }
  // position right after sender s has been added to the stream
  int pos_after_sender(int s) const {
    if (s == 0) return 0;
    int l = (s - 1) / (H + mu), r = (s - 1) % (H + mu);
    return r < H ? 2 * l + 1 : 2 * l + 2;
  }
};

}  // namespace pahq
