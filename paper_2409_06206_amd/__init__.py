"""MI355X-native Group Shifted Window Attention (GSWA) layer, forward and backward.

``paper_2409_06206_amd.gswa`` is the thin binding over the C-ABI HIP library;
``paper_2409_06206_amd.synth`` draws the seeded synthetic inputs.  Importing the
package loads nothing; the HIP library is loaded on the first call and its
absence is an error, never a fallback.
"""
