"""Device-resident experience replay and Q-learning train step for MI355X (gfx950).

The GPU library is loaded lazily by `paper_1801_03138_amd.binding`; importing the
package itself (for example to reach `synth`) touches no native code.
"""
