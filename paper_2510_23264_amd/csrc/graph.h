// Node / edge numbering of the computational graph (host side).
// Paper, Appendix "Preliminaries", Circuit Discovery: nodes are attention heads
// and MLP layers plus embedding and unembedding; a node reads the sum of its
// predecessors.  Head inputs are split into query / key / value receivers.
#pragma once
#include <stdint.h>

namespace pahq {

struct GraphDims {
  int L, H, mu, Ns, Nr;
  GraphDims() : L(0), H(0), mu(0), Ns(0), Nr(0) {}
  GraphDims(int L_, int H_, bool mlp) : L(L_), H(H_), mu(mlp ? 1 : 0) {
    Ns = 1 + L * (H + mu);
    Nr = L * (3 * H + mu) + 1;
  }
  int head(int l, int h) const { return 1 + l * (H + mu) + h; }
  int mlp(int l) const { return 1 + l * (H + mu) + H; }
  int headin(int l, int h, int c) const { return l * (3 * H + mu) + 3 * h + c; }
  int mlpin(int l) const { return l * (3 * H + mu) + 3 * H; }
  int out() const { return Nr - 1; }
  // kind: 0 headin, 1 mlpin, 2 out
  void receiver_info(int r, int& kind, int& l, int& h, int& c) const {
    if (r == Nr - 1) { kind = 2; l = L; h = c = -1; return; }
    l = r / (3 * H + mu);
    int q = r % (3 * H + mu);
    if (q < 3 * H) { kind = 0; h = q / 3; c = q % 3; } else { kind = 1; h = c = -1; }
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
