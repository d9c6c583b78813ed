"""MI355X-native forward pass of stacked LSTM / GRU networks (persistent wavefront execution).

The compiled library is loaded lazily by :mod:`paper_2307_11339_amd.rnn`; importing this
package (for example for :mod:`paper_2307_11339_amd.workloads`) touches no GPU code.
"""
